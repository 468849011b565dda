"""Operands stored in slabs of 128 contraction bytes (LLMQ_LAYOUT_SLABS of llmq_fp8_gemm, LLMQ_SLAB_COPIES of the
linear calls): a layout only, so every result must be the bytes of the plain layout, and the slab copies in the
workspace must be the plain transposed copies rearranged."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_15306_amd import llmq, synth
from gpu_common import DEV, GEMM_TOL, gpu_amax
from test_gpu_gemm import _rand_codes, _scales, _sample_positions

pytestmark = pytest.mark.gpu


def to_slabs(t: torch.Tensor) -> torch.Tensor:
    """[rows, T] -> [T / 128, rows, 128]."""
    rows, T = t.shape
    return t.view(rows, T // 128, 128).permute(1, 0, 2).contiguous()


def from_slabs(t: torch.Tensor, rows: int, T: int) -> torch.Tensor:
    return t.view(T // 128, rows, 128).permute(1, 0, 2).reshape(rows, T)


@pytest.mark.parametrize("R,C,T", [(256, 256, 512), (512, 384, 1152), (384, 768, 256), (128, 128, 128), (1024, 1280, 2176),
                                   (48, 80, 384), (33, 17, 128)])
@pytest.mark.parametrize("fa,fb", [(0, 0), (1, 0), (0, 1)])
def test_contraction_on_slab_operands_gives_the_same_bytes(R, C, T, fa, fb):
    """Tuned tiles of several shapes and the generic kernel (last two shapes); either operand or both in slabs,
    also next to a T-major one, with and without accumulation, fused absmax included."""
    print("R=%d C=%d T=%d fa=%d fb=%d" % (R, C, T, fa, fb), flush=True)
    A = torch.from_numpy(_rand_codes((R, T), fa, 3)).to(DEV)
    B = torch.from_numpy(_rand_codes((C, T), fb, 4)).to(DEV)
    dsa, dsb = _scales(2.0, 0.5)
    forms_a = {0: A, 1: A.t().contiguous(), 2: to_slabs(A)}
    forms_b = {0: B, 1: B.t().contiguous(), 2: to_slabs(B)}
    base = torch.randn((R, C), device=DEV).to(torch.bfloat16)

    def run(la, lb, accumulate):
        c = base.clone() if accumulate else torch.full((R, C), float("nan"), dtype=torch.bfloat16, device=DEV)
        am = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
        llmq.llmq_fp8_gemm(forms_a[la], fa, la, forms_b[lb], fb, lb, dsa, dsb, c, accumulate, am)
        return c, am

    for accumulate in (False, True):
        want_c, want_am = run(0, 0, accumulate)
        for la, lb in ((2, 0), (0, 2), (2, 2), (2, 1), (1, 2)):
            c, am = run(la, lb, accumulate)
            assert torch.equal(c.view(torch.int16), want_c.view(torch.int16)), (la, lb, accumulate)
            assert torch.equal(am, want_am), (la, lb, accumulate)


@pytest.mark.parametrize("cfg_i,li,extra", [(1, 0, 0), (3, 1, 0), (5, 0, llmq.SHARE_TILES), (2, 3, 0)])
def test_linear_calls_with_slab_copies(cfg_i, li, extra):
    """The three linear calls with and without LLMQ_SLAB_COPIES (config 5's qkv projection also with shared tiles):
    same outputs, same scales, the row-major copies the same bytes, the transposed copies the same bytes once taken
    out of their slabs; and reuse of slab copies across calls (the weight gradient runs on copies the other two
    calls left)."""
    cfg = synth.CONFIGS[cfg_i]
    lin = cfg.linears[li]
    M, K, N = cfg.M, lin.K, lin.N
    print("config %d %s M=%d K=%d N=%d" % (cfg_i, lin.name, M, K, N), flush=True)
    X, W, dY = synth.make_x(cfg, li, device=DEV), synth.make_w(cfg, li, device=DEV), synth.make_dy(cfg, li, device=DEV)
    nbytes = llmq.llmq_fp8_linear_workspace_bytes_shared(M, N, K)
    offs = llmq.llmq_fp8_linear_workspace_offsets(M, N, K)

    def run(flags):
        ws = torch.full((nbytes,), 0xEE, dtype=torch.uint8, device=DEV)
        sx, sw, sd = (torch.zeros(1, dtype=torch.float32, device=DEV) for _ in range(3))
        Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
        dX = torch.full((M, K), float("nan"), dtype=torch.bfloat16, device=DEV)
        dW = torch.full((N, K), float("nan"), dtype=torch.bfloat16, device=DEV)
        ay, adx = (torch.full((1,), -1.0, dtype=torch.float32, device=DEV) for _ in range(2))
        llmq.llmq_fp8_linear_fwd(X, W, M, N, K, sx, sw, Y, ay, ws, flags | llmq.JIT_X | llmq.JIT_W)
        llmq.llmq_fp8_linear_dgrad(dY, None, M, N, K, sd, sw, llmq.E5M2, dX, adx, ws, flags | llmq.JIT_DY | llmq.REUSE_W)
        llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, sd, sx, llmq.E5M2, dW, False, ws, flags | llmq.REUSE_X | llmq.REUSE_DY)
        torch.cuda.synchronize()
        return dict(Y=Y, dX=dX, dW=dW, ay=ay, adx=adx, sx=sx, sw=sw, sd=sd, ws=ws)

    plain = run(extra)
    slabs = run(extra | llmq.SLAB_COPIES)
    for k in ("Y", "dX", "dW"):
        assert torch.equal(plain[k].view(torch.int16), slabs[k].view(torch.int16)), k
    for k in ("ay", "adx", "sx", "sw", "sd"):
        assert torch.equal(plain[k], slabs[k]), k
    copy = lambda r, i, rows, cols: r["ws"][offs[i]:offs[i] + rows * cols]
    # row-major copies: Xq [M,K], Wq [N,K], dYq [M,N]
    for i, (rows, cols) in ((0, (M, K)), (2, (N, K)), (4, (M, N))):
        assert torch.equal(copy(plain, i, rows, cols), copy(slabs, i, rows, cols)), i
    # transposed copies of x [rows, cols]: [cols, rows], in slabs where the quantizer's tile kernel takes the tensor
    any_slabs = False
    for i, (rows, cols) in ((1, (M, K)), (3, (N, K)), (5, (M, N))):
        want = copy(plain, i, rows, cols).view(cols, rows)
        got = copy(slabs, i, rows, cols)
        if rows % 128 == 0 and cols % 256 == 0:
            any_slabs = True
            got = from_slabs(got, cols, rows)
            assert not torch.equal(copy(slabs, i, rows, cols), copy(plain, i, rows, cols)) or rows == 128
        assert torch.equal(got.reshape(cols, rows), want), i
    assert any_slabs == (cfg_i != 1 or (M % 128 == 0 and K % 256 == 0))


@pytest.mark.parametrize("rows,cols", [(128, 256), (384, 768), (4096, 3072)])
@pytest.mark.parametrize("fmt", [0, 1])
def test_quantize_with_the_transposed_copy_in_slabs(rows, cols, fmt):
    """llmq_quantize_fp8_slabs against the oracle: q bit for bit, q_t bit for bit once taken out of its slabs."""
    x = (torch.randn((rows, cols), device=DEV) * 3).to(torch.bfloat16)
    scale = 17.0
    ds = torch.tensor([scale], dtype=torch.float32, device=DEV)
    q = torch.full((rows, cols), 0xEE, dtype=torch.uint8, device=DEV)
    qt = torch.full((rows * cols,), 0xEE, dtype=torch.uint8, device=DEV)
    llmq.llmq_quantize_fp8_slabs(x, ds, fmt, q, qt)
    want_q, want_qt = oracle.quantize(x.view(torch.int16).cpu().numpy().view(np.uint16), scale, fmt)
    assert np.array_equal(q.cpu().numpy(), want_q)
    assert np.array_equal(from_slabs(qt, cols, rows).cpu().numpy(), want_qt)
    with pytest.raises(llmq.LlmqError):
        llmq.llmq_quantize_fp8_slabs(x[:rows - 8].contiguous(), ds, fmt, q[:rows - 8].contiguous(), qt[:(rows - 8) * cols].contiguous())


# ---- the producers that write FP8 directly, with the transposed copy in slabs ----

def _bits(t):
    return synth.bf16_bits(t)


@pytest.mark.parametrize("M,I", [(128, 256), (384, 768), (256, 2048)])
@pytest.mark.parametrize("fmt", [0, 1])
def test_swiglu_fp8_with_the_transposed_copy_in_slabs(M, I, fmt):
    """llmq_swiglu_fwd_fp8_slabs against the oracle: h and q bit for bit, q_t bit for bit once taken out of its
    slabs; shapes that are not whole tiles are refused."""
    print("swiglu fwd_fp8_slabs M=%d I=%d fmt=%d" % (M, I, fmt), flush=True)
    g = torch.Generator(device="cpu").manual_seed(77 + M + I)
    gu = torch.cat([torch.randn(M, I, generator=g) * 2.0, torch.randn(M, I, generator=g) * 1.5], dim=1).to(torch.bfloat16)
    want_h = oracle.swiglu_fwd(_bits(gu))
    sc = oracle.scale(oracle.amax_bf16(want_h), fmt)
    want_q, want_qt = oracle.quantize(want_h, sc, fmt)
    gud = gu.to(DEV)
    ds = torch.tensor([float(sc)], dtype=torch.float32, device=DEV)
    for want_y in (True, False):
        q = torch.full((M, I), 0xEE, dtype=torch.uint8, device=DEV)
        qt = torch.full((M * I,), 0xEE, dtype=torch.uint8, device=DEV)
        h = torch.full((M, I), -7.0, dtype=torch.bfloat16, device=DEV) if want_y else None
        llmq.llmq_swiglu_fwd_fp8_slabs(gud, ds, fmt, q, qt, h)
        assert np.array_equal(q.cpu().numpy(), want_q)
        assert np.array_equal(from_slabs(qt, I, M).cpu().numpy(), want_qt)
        if want_y:
            assert np.array_equal(_bits(h), want_h)
    with pytest.raises(llmq.LlmqError):
        llmq.llmq_swiglu_fwd_fp8_slabs(gud[:M - 16].contiguous(), ds, fmt, q[:M - 16].contiguous(),
                                       qt[:(M - 16) * I].contiguous(), None)


@pytest.mark.parametrize("M,C", [(128, 256), (384, 768), (256, 3584)])
@pytest.mark.parametrize("fmt", [0, 1])
def test_rmsnorm_recompute_with_the_transposed_copy_in_slabs(M, C, fmt):
    """llmq_rmsnorm_apply_fp8_slabs against the oracle, as above."""
    print("rmsnorm apply_fp8_slabs M=%d C=%d fmt=%d" % (M, C, fmt), flush=True)
    g = torch.Generator(device="cpu").manual_seed(55 + M + C)
    res = (torch.randn(M, C, generator=g) * 1.3).to(torch.bfloat16)
    w = (1.0 + 0.2 * torch.randn(C, generator=g)).to(torch.bfloat16)
    rb, wb = _bits(res), _bits(w)
    rstd = oracle.rms_rstd(rb, 1e-6).astype(np.float32)
    want_y = oracle.rmsnorm_apply(rb, wb, rstd)
    sc = oracle.scale(oracle.amax_bf16(want_y), fmt)
    want_q, want_qt = oracle.quantize(want_y, sc, fmt)
    res_d, w_d, rstd_d = res.to(DEV), w.to(DEV), torch.from_numpy(rstd).to(DEV)
    ds = torch.tensor([float(sc)], dtype=torch.float32, device=DEV)
    for with_y in (True, False):
        q = torch.full((M, C), 0xEE, dtype=torch.uint8, device=DEV)
        qt = torch.full((M * C,), 0xEE, dtype=torch.uint8, device=DEV)
        y = torch.full((M, C), -7.0, dtype=torch.bfloat16, device=DEV) if with_y else None
        llmq.llmq_rmsnorm_apply_fp8_slabs(res_d, w_d, rstd_d, ds, fmt, q, qt, y)
        assert np.array_equal(q.cpu().numpy(), want_q)
        assert np.array_equal(from_slabs(qt, C, M).cpu().numpy(), want_qt)
        if with_y:
            assert np.array_equal(_bits(y), want_y)
    with pytest.raises(llmq.LlmqError):
        llmq.llmq_rmsnorm_apply_fp8_slabs(res_d[:, :C - 8].contiguous(), w_d[:C - 8].contiguous(), rstd_d, ds, fmt,
                                          q[:, :C - 8].contiguous(), qt[:M * (C - 8)].contiguous(), None)


def test_slab_copies_of_a_producer_feed_the_linear_calls():
    """Recompute mode end to end under LLMQ_SLAB_COPIES: the copies llmq_swiglu_fwd_fp8_slabs writes straight into
    the workspace of the down projection are the ones the linear call would have made from h, so forward and
    weight-gradient calls that reuse them give the same bytes."""
    M, I, N = 256, 512, 384
    g = torch.Generator(device="cpu").manual_seed(4243)
    gu = torch.cat([torch.randn(M, I, generator=g) * 2.0, torch.randn(M, I, generator=g) * 1.5], dim=1).to(torch.bfloat16).to(DEV)
    W = (torch.randn(N, I, generator=g) * 0.02).to(torch.bfloat16).to(DEV)
    dY = (torch.randn(M, N, generator=g) * 1e-3).to(torch.bfloat16).to(DEV)
    h = torch.empty((M, I), dtype=torch.bfloat16, device=DEV)
    a = torch.empty(1, device=DEV)
    s_h = torch.empty(1, device=DEV)
    llmq.llmq_swiglu_fwd(gu, h, 0, a, s_h, torch.empty(llmq.llmq_swiglu_workspace_bytes(M, I), dtype=torch.uint8, device=DEV))
    _, s_w = gpu_amax(W, 0)
    _, s_dy = gpu_amax(dY, 1)
    ws_bytes = llmq.llmq_fp8_linear_workspace_bytes(M, N, I)
    off = llmq.llmq_fp8_linear_workspace_offsets(M, N, I)
    flags = llmq.SLAB_COPIES

    def run(reuse):
        ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=DEV)
        y = torch.zeros((M, N), dtype=torch.bfloat16, device=DEV)
        dW = torch.zeros((N, I), dtype=torch.bfloat16, device=DEV)
        if reuse:
            llmq.llmq_swiglu_fwd_fp8_slabs(gu, s_h, 0, ws[off[0]:off[0] + M * I], ws[off[1]:off[1] + M * I], None)
            llmq.llmq_fp8_linear_fwd(None, W, M, N, I, s_h, s_w, y, None, ws, flags=flags | llmq.REUSE_X)
        else:
            llmq.llmq_fp8_linear_fwd(h, W, M, N, I, s_h, s_w, y, None, ws, flags=flags)
        llmq.llmq_fp8_linear_wgrad(dY, None, M, N, I, s_dy, s_h, 1, dW, False, ws, flags=flags | llmq.REUSE_X)
        return ws, y, dW

    ws1, y1, dW1 = run(False)
    ws2, y2, dW2 = run(True)
    assert torch.equal(ws1, ws2) and torch.equal(y1, y2) and torch.equal(dW1, dW2)


def test_producers_at_full_size_write_the_same_copies_in_slabs():
    """Config 5 (32B-class) SwiGLU and RMSNorm recompute at the benchmark's sizes: the slab variants against the
    plain ones on the GPU (those are compared with the oracle, whole tensors, in their own tests)."""
    cfg = synth.CONFIGS[5]
    M, I = synth.swiglu_dims(cfg)
    print("full-size swiglu slabs M=%d I=%d" % (M, I), flush=True)
    gu = synth.make_gu(cfg, device=DEV)
    ds = torch.tensor([3.0], dtype=torch.float32, device=DEV)
    q1 = torch.empty((M, I), dtype=torch.uint8, device=DEV)
    qt1 = torch.empty((I, M), dtype=torch.uint8, device=DEV)
    q2 = torch.full((M, I), 0xEE, dtype=torch.uint8, device=DEV)
    qt2 = torch.full((M * I,), 0xEE, dtype=torch.uint8, device=DEV)
    llmq.llmq_swiglu_fwd_fp8(gu, ds, 0, q1, qt1, None)
    llmq.llmq_swiglu_fwd_fp8_slabs(gu, ds, 0, q2, qt2, None)
    assert torch.equal(q1, q2) and torch.equal(from_slabs(qt2, I, M), qt1)
    del gu, q1, qt1, q2, qt2
    torch.cuda.empty_cache()
    res, x, w = synth.make_norm_inputs(cfg, device=DEV)
    M, C = res.shape
    print("full-size rmsnorm slabs M=%d C=%d" % (M, C), flush=True)
    rstd = torch.rand(M, device=DEV) + 0.5
    q1 = torch.empty((M, C), dtype=torch.uint8, device=DEV)
    qt1 = torch.empty((C, M), dtype=torch.uint8, device=DEV)
    q2 = torch.full((M, C), 0xEE, dtype=torch.uint8, device=DEV)
    qt2 = torch.full((M * C,), 0xEE, dtype=torch.uint8, device=DEV)
    llmq.llmq_rmsnorm_apply_fp8(res, w, rstd, ds, 0, q1, qt1, None)
    llmq.llmq_rmsnorm_apply_fp8_slabs(res, w, rstd, ds, 0, q2, qt2, None)
    assert torch.equal(q1, q2) and torch.equal(from_slabs(qt2, C, M), qt1)
