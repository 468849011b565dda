"""GPU parity: the FP8 contraction and the three linear-layer calls against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_15306_amd import llmq, synth
from gpu_common import (DEV, GEMM_TOL, f32_bits, np_f32_bits, gpu_amax, gpu_quantize, oracle_quantized,
                        bf16_to_f64, assert_gemm_close)

pytestmark = pytest.mark.gpu


def _rand_codes(shape, fmt, seed):
    """Random finite FP8 codes with moderate magnitudes (exponent field in the middle of the range)."""
    rng = np.random.default_rng(seed)
    if fmt == 0:
        e = rng.integers(3, 11, size=shape)
        m = rng.integers(0, 8, size=shape)
        c = (e << 3) | m
    else:
        e = rng.integers(10, 20, size=shape)
        m = rng.integers(0, 4, size=shape)
        c = (e << 2) | m
    c |= rng.integers(0, 2, size=shape) << 7
    return c.astype(np.uint8)


def _scales(sa, sb):
    return (torch.tensor([sa], dtype=torch.float32, device=DEV), torch.tensor([sb], dtype=torch.float32, device=DEV))


def _run_gemm(A, fa, B, fb, sa, sb, accumulate=False, c_init=None, want_amax=False):
    Ad, Bd = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    dsa, dsb = _scales(sa, sb)
    c = torch.full((A.shape[0], B.shape[0]), float("nan"), dtype=torch.bfloat16, device=DEV) if c_init is None else c_init.clone()
    am = torch.full((1,), -1.0, dtype=torch.float32, device=DEV) if want_amax else None
    llmq.llmq_fp8_gemm_tn(Ad, fa, Bd, fb, dsa, dsb, c, accumulate, am)
    return c, am


# generic path: odd shapes, ragged K; tuned path: multiples of 256 x 256 x 128 (odd and even K steps)
GEMM_SHAPES = [(1, 1, 1), (5, 3, 7), (16, 16, 128), (33, 17, 130), (100, 136, 72), (48, 40, 1000),
               (256, 256, 128), (256, 256, 256), (256, 512, 384), (512, 256, 640), (768, 1024, 512)]


@pytest.mark.parametrize("R,C,T", GEMM_SHAPES)
@pytest.mark.parametrize("fa,fb", [(0, 0), (1, 0), (0, 1), (1, 1)])
def test_gemm_tn_within_tolerance(R, C, T, fa, fb):
    print("gemm R=%d C=%d T=%d fa=%d fb=%d" % (R, C, T, fa, fb), flush=True)
    A = _rand_codes((R, T), fa, 11 * R + T + fa)
    B = _rand_codes((C, T), fb, 13 * C + T + fb + 1)
    sa, sb = 3.7, 0.61
    c, am = _run_gemm(A, fa, B, fb, sa, sb, want_amax=True)
    y, S = oracle.gemm_tn(A, fa, B, fb, sa, sb)
    assert_gemm_close(c, y, S, "gemm")
    # fused output absmax == absmax of the BF16 result the kernel wrote, bit for bit
    a2, _ = gpu_amax(c.reshape(-1), 0, want_scale=False)
    assert f32_bits(am) == f32_bits(a2)
    assert am.item() == c.float().abs().max().item()
    # determinism
    c2, _ = _run_gemm(A, fa, B, fb, sa, sb)
    assert torch.equal(c2.view(torch.int16), c.view(torch.int16))


@pytest.mark.parametrize("R,C,T", [(256, 256, 256), (512, 768, 384), (48, 40, 1000)])
def test_fused_absmax_reports_a_nan_output(R, C, T):
    """One NaN code in A makes one output row NaN; the fused absmax of the tuned kernel (first two shapes) and
    of the generic one (last) must then be the canonical NaN that llmq_amax reports for the stored tensor,
    and an Inf output (E5M2 Inf code) must give +Inf."""
    A = _rand_codes((R, T), 0, 91)
    B = _rand_codes((C, T), 0, 92)
    A[R // 2 + 1, T // 3] = 0x7F                          # E4M3 NaN
    c, am = _run_gemm(A, 0, B, 0, 1.5, 0.8, want_amax=True)
    a2, _ = gpu_amax(c.reshape(-1), 0, want_scale=False)
    assert torch.isnan(c[R // 2 + 1]).all() and not torch.isnan(c[R // 2]).any()
    assert f32_bits(am) == f32_bits(a2) == 0x7FC00000
    A5 = _rand_codes((R, T), 1, 93)
    A5[R - 1, 0] = 0x7C                                   # E5M2 +Inf
    B[:, 0] = 0x38                                        # E4M3 1.0: the Inf row stays Inf, no 0 * Inf
    c, am = _run_gemm(A5, 1, B, 0, 1.5, 0.8, want_amax=True)
    a2, _ = gpu_amax(c.reshape(-1), 0, want_scale=False)
    assert torch.isinf(c[R - 1]).all()
    assert f32_bits(am) == f32_bits(a2) == 0x7F800000


@pytest.mark.parametrize("tile", ["4x4", "4x3", "4x2", "3x4", "3x3", "3x2", "2x4", "2x3", "2x2"])
def test_every_tuned_tile_shape(tile, monkeypatch):
    """Each wave-tile instantiation of the tuned kernel, forced through the tuning override, on a
    problem of 2 x 3 workgroup tiles with an odd number of K steps, mixed formats, fused absmax."""
    ni, nj = int(tile[0]), int(tile[2])
    R, C, T = 2 * 64 * ni, 3 * 64 * nj, 640
    print("tile %s R=%d C=%d T=%d" % (tile, R, C, T), flush=True)
    monkeypatch.setenv("LLMQ_GEMM_TILE", tile)
    A = _rand_codes((R, T), 1, 41 + ni)
    B = _rand_codes((C, T), 0, 43 + nj)
    c, am = _run_gemm(A, 1, B, 0, 1.9, 0.7, want_amax=True)
    monkeypatch.delenv("LLMQ_GEMM_TILE")
    y, S = oracle.gemm_tn(A, 1, B, 0, 1.9, 0.7)
    assert_gemm_close(c, y, S, "tile " + tile)
    assert am.item() == c.float().abs().max().item()
    c2, _ = _run_gemm(A, 1, B, 0, 1.9, 0.7)          # the shape the library picks by itself: same bytes
    assert torch.equal(c2.view(torch.int16), c.view(torch.int16))


@pytest.mark.parametrize("R,C,T", [(33, 17, 130), (256, 512, 384)])
def test_gemm_accumulate_in_bf16(R, C, T):
    A = _rand_codes((R, T), 1, 5)
    B = _rand_codes((C, T), 0, 6)
    sa, sb = 2.0, 0.5
    g = torch.Generator().manual_seed(3)
    c0 = (torch.randn((R, C), generator=g) * 50).to(torch.bfloat16).to(DEV)
    c, _ = _run_gemm(A, 1, B, 0, sa, sb, accumulate=True, c_init=c0)
    y, S = oracle.gemm_tn(A, 1, B, 0, sa, sb)
    want = bf16_to_f64(c0) + y
    got = bf16_to_f64(c)
    # one extra BF16 rounding of the sum on top of the GEMM tolerance
    assert np.all(np.abs(got - want) <= GEMM_TOL * S + 2.0 ** -8 * np.abs(want))


def test_accumulation_is_one_rounding_of_the_exact_sum_in_every_tile_shape():
    """Small-integer operands and power-of-two scales: the binary32 contraction, its de-scaling and the addition
    of the old BF16 value are all exact, so `accumulate` must give RNE-to-BF16 of the exact sum, bit for bit,
    whatever wave tile computes it (each has its own staging geometry in the epilogue), with the fused absmax that
    of the stored result; run twice per shape: the second call accumulates onto the first."""
    import os
    R, C, T = 768, 1536, 384                      # multiples of 128, 192 and 256: every tile shape divides them
    rng = np.random.default_rng(77)
    Ai, Bi = rng.integers(-3, 4, size=(R, T)), rng.integers(-3, 4, size=(C, T))
    to_bits = lambda v: synth.bf16_bits(torch.from_numpy(v.astype(np.float32)).to(torch.bfloat16))
    A = oracle.quantize(to_bits(Ai), 1.0, 1)[0]
    B = oracle.quantize(to_bits(Bi), 1.0, 0)[0]
    dec_a, dec_b = oracle.decode_table(1), oracle.decode_table(0)
    assert np.array_equal(dec_a[A], Ai.astype(np.float64)) and np.array_equal(dec_b[B], Bi.astype(np.float64))
    y = (Ai @ Bi.T).astype(np.float64) / 2.0       # scales 4 and 0.5: de-scaling multiplies by 1 / 2
    Ad, Bd = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    dsa, dsb = _scales(4.0, 0.5)
    g = torch.Generator().manual_seed(11)
    c0 = (torch.round(torch.randn((R, C), generator=g) * 160) / 4).to(torch.bfloat16)      # multiples of 1/4
    rne = lambda v: torch.from_numpy(v).to(torch.float32).to(torch.bfloat16)     # exact in binary32, one rounding
    want1 = rne(bf16_to_f64(c0) + y)
    want2 = rne(bf16_to_f64(want1) + y)
    assert np.all(np.abs(bf16_to_f64(c0) + y) < 2.0 ** 14)       # 16 bits above the quarter: the binary32 sum is exact
    try:
        for tile in ["4x4", "2x2", "4x3", "3x4", "3x3", "4x2", "2x4", "3x2", "2x3"]:
            os.environ["LLMQ_GEMM_TILE"] = tile
            c = c0.to(DEV).clone()
            am = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
            llmq.llmq_fp8_gemm_tn(Ad, 1, Bd, 0, dsa, dsb, c, True, am)
            assert torch.equal(c.cpu().view(torch.int16), want1.view(torch.int16)), "tile %s, first call" % tile
            assert am.item() == want1.float().abs().max().item(), tile
            llmq.llmq_fp8_gemm_tn(Ad, 1, Bd, 0, dsa, dsb, c, True, am)
            assert torch.equal(c.cpu().view(torch.int16), want2.view(torch.int16)), "tile %s, second call" % tile
            assert am.item() == want2.float().abs().max().item(), tile
    finally:
        os.environ.pop("LLMQ_GEMM_TILE", None)


@pytest.mark.parametrize("M,K,N", [(5, 7, 3), (40, 32, 24), (256, 128, 256)])
def test_integer_inputs_give_exact_products(M, K, N):
    """Lossless inputs (small integers, absmax 7): every GEMM result is an exact small integer."""
    rng = np.random.default_rng(M + K + N)

    def ints(shape):
        v = rng.integers(-2, 3, size=shape).astype(np.float32)
        v[tuple(rng.integers(0, s) for s in shape)] = 7.0
        return torch.from_numpy(v).to(torch.bfloat16)

    X, W, dY = ints((M, K)), ints((N, K)), ints((M, N))
    Xd, Wd, dYd = X.to(DEV), W.to(DEV), dY.to(DEV)
    ws = torch.empty(llmq.llmq_fp8_linear_workspace_bytes(M, N, K), dtype=torch.uint8, device=DEV)
    _, sx = gpu_amax(Xd, 0)
    _, sw = gpu_amax(Wd, 0)
    _, sd = gpu_amax(dYd, 1)
    assert (sx.item(), sw.item(), sd.item()) == (64.0, 64.0, 8192.0)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    dX = torch.empty((M, K), dtype=torch.bfloat16, device=DEV)
    dW = torch.empty((N, K), dtype=torch.bfloat16, device=DEV)
    llmq.llmq_fp8_linear_fwd(Xd, Wd, M, N, K, sx, sw, Y, None, ws)
    llmq.llmq_fp8_linear_dgrad(dYd, Wd, M, N, K, sd, sw, 1, dX, None, ws, llmq.REUSE_W)
    llmq.llmq_fp8_linear_wgrad(dYd, Xd, M, N, K, sd, sx, 1, dW, False, ws, llmq.REUSE_X | llmq.REUSE_DY)
    Xi, Wi, Di = X.double().numpy(), W.double().numpy(), dY.double().numpy()
    assert np.array_equal(bf16_to_f64(Y), Xi @ Wi.T)
    assert np.array_equal(bf16_to_f64(dX), Di @ Wi)
    assert np.array_equal(bf16_to_f64(dW), Di.T @ Xi)


def _linear_case(cfg, li, M=None, fmt_dy=1, K=None, N=None):
    x = synth.make_x(cfg, li, device="cpu", M=M)
    w = synth.make_w(cfg, li, device="cpu")
    dy = synth.make_dy(cfg, li, device="cpu", M=M)
    if K is not None:
        x, w = x[:, :K].contiguous(), w[:, :K].contiguous()
    if N is not None:
        w, dy = w[:N].contiguous(), dy[:, :N].contiguous()
    return x, w, dy


@pytest.mark.parametrize("shape", synth.small_cases())
@pytest.mark.parametrize("fmt_dy", [1, 0])
def test_linear_fwd_dgrad_wgrad_full_compare(shape, fmt_dy):
    """Whole outputs of the three calls against the oracle on config-1 style inputs, every workspace
    copy bit-exact, every reuse flag exercised."""
    M, K, N = shape
    print("linear M=%d K=%d N=%d fmt_dy=%d" % (M, K, N, fmt_dy), flush=True)
    cfg = synth.CONFIGS[1]
    x, w, dy = _linear_case(cfg, 0, M=M, K=K if K <= 512 else None, N=N if N <= 1024 else None)
    if x.shape[1] != K or w.shape[0] != N:      # shapes beyond config 1's tensor: draw fresh ones
        g = torch.Generator().manual_seed(M * 7 + K * 3 + N)
        x = torch.randn((M, K), generator=g).to(torch.bfloat16)
        w = (torch.randn((N, K), generator=g) * 0.02).to(torch.bfloat16)
        dy = (torch.randn((M, N), generator=g) * 1e-3).to(torch.bfloat16)
    ax, sx, xq, xqt = oracle_quantized(x, 0)
    aw, sw, wq, wqt = oracle_quantized(w, 0)
    ad, sd, dq, dqt = oracle_quantized(dy, fmt_dy)
    xd, wd, dyd = x.to(DEV), w.to(DEV), dy.to(DEV)
    _, gsx = gpu_amax(xd, 0)
    _, gsw = gpu_amax(wd, 0)
    _, gsd = gpu_amax(dyd, fmt_dy)
    assert [f32_bits(t) for t in (gsx, gsw, gsd)] == [np_f32_bits(v) for v in (sx, sw, sd)]
    nbytes = llmq.llmq_fp8_linear_workspace_bytes(M, N, K)
    offs = llmq.llmq_fp8_linear_workspace_offsets(M, N, K)
    ws = torch.full((nbytes,), 0x55, dtype=torch.uint8, device=DEV)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    dX = torch.empty((M, K), dtype=torch.bfloat16, device=DEV)
    dW = torch.empty((N, K), dtype=torch.bfloat16, device=DEV)
    amax_y = torch.zeros(1, dtype=torch.float32, device=DEV)
    amax_dx = torch.zeros(1, dtype=torch.float32, device=DEV)
    llmq.llmq_fp8_linear_fwd(xd, wd, M, N, K, gsx, gsw, Y, amax_y, ws)
    llmq.llmq_fp8_linear_dgrad(dyd, None, M, N, K, gsd, gsw, fmt_dy, dX, amax_dx, ws, llmq.REUSE_W)
    llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, gsd, gsx, fmt_dy, dW, False, ws, llmq.REUSE_X | llmq.REUSE_DY)
    wsh = ws.cpu().numpy()
    for off, want in zip(offs, (xq, xqt, wq, wqt, dq, dqt)):
        assert np.array_equal(wsh[off:off + want.size].reshape(want.shape), want)
    y, S = oracle.gemm_tn(xq, 0, wq, 0, sx, sw)
    assert_gemm_close(Y, y, S, "fwd")
    y, S = oracle.gemm_tn(dq, fmt_dy, wqt, 0, sd, sw)
    assert_gemm_close(dX, y, S, "dgrad")
    y, S = oracle.gemm_tn(dqt, fmt_dy, xqt, 0, sd, sx)
    assert_gemm_close(dW, y, S, "wgrad")
    assert amax_y.item() == Y.float().abs().max().item()
    assert amax_dx.item() == dX.float().abs().max().item()
    # without reuse flags the backward calls quantize for themselves and give the same bytes
    ws2 = torch.full((nbytes,), 0x33, dtype=torch.uint8, device=DEV)
    dX2, dW2 = torch.empty_like(dX), torch.empty_like(dW)
    llmq.llmq_fp8_linear_dgrad(dyd, wd, M, N, K, gsd, gsw, fmt_dy, dX2, None, ws2, 0)
    llmq.llmq_fp8_linear_wgrad(dyd, xd, M, N, K, gsd, gsx, fmt_dy, dW2, False, ws2, 0)
    assert torch.equal(dX2.view(torch.int16), dX.view(torch.int16))
    assert torch.equal(dW2.view(torch.int16), dW.view(torch.int16))
    # gradient accumulation: dW += on top of the previous result
    llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, gsd, gsx, fmt_dy, dW2, True, ws2, llmq.REUSE_X | llmq.REUSE_DY)
    want2 = 2.0 * y
    assert np.all(np.abs(bf16_to_f64(dW2) - want2) <= 2 * GEMM_TOL * S + 2.0 ** -8 * np.abs(want2))


def _sample_positions(R, C, n, seed, tile=256):
    rng = np.random.default_rng(seed)
    rr = rng.integers(0, R, n)
    cc = rng.integers(0, C, n)
    # plus full tile-boundary rows and columns (first/last row of interior tiles), subsampled
    rows = [0, R - 1] + ([tile - 1, tile] if R > tile else [])
    cols = [0, C - 1] + ([tile - 1, tile] if C > tile else [])
    er, ec = [], []
    for r in rows:
        cs = np.unique(np.concatenate([np.arange(0, C, max(1, C // 257)), [C - 1]]))
        er.append(np.full(cs.shape, r)); ec.append(cs)
    for c in cols:
        rs = np.unique(np.concatenate([np.arange(0, R, max(1, R // 257)), [R - 1]]))
        er.append(rs); ec.append(np.full(rs.shape, c))
    return np.concatenate([rr] + er), np.concatenate([cc] + ec)


# Every linear of configs 2-5 with explicit scales (llmq_amax first) and with just-in-time scaling inside the
# calls, which is the launch sequence bench.py times; E5M2 gradients as in the benchmark configurations, plus
# one linear per config with E4M3 gradients (Section 5, Scenario 1 of the paper tried both).
FULL_SIZE_CASES = [(c, l, jit, 1) for c in (2, 3, 4, 5) for l in range(4) for jit in (False, True)] + \
                  [(2, 1, True, 0), (3, 2, True, 0), (4, 0, True, 0), (5, 3, True, 0), (3, 3, False, 0)]


@pytest.mark.parametrize("cfg_i,li,jit,fmt_dy", FULL_SIZE_CASES)
def test_full_size_linears_on_sampled_outputs(cfg_i, li, jit, fmt_dy):
    """The benchmark configurations' shapes; with jit the three calls run exactly as bench.py's step runs them
    (LLMQ_JIT_X | LLMQ_JIT_W, LLMQ_JIT_DY | LLMQ_REUSE_W, LLMQ_REUSE_X | LLMQ_REUSE_DY: the scales are outputs of
    the calls), without it the scales come from llmq_amax.  Either way the scales must be the oracle's bit
    for bit, the six quantized copies are compared in full, and the oracle computes >= 4096 random outputs
    plus tile-boundary rows and columns of each of the three GEMMs with full-length dot products."""
    cfg = synth.CONFIGS[cfg_i]
    lin = cfg.linears[li]
    M, K, N = cfg.M, lin.K, lin.N
    print("full-size config %d %s M=%d K=%d N=%d jit=%d fmt_dy=%d" % (cfg_i, lin.name, M, K, N, jit, fmt_dy), flush=True)
    xd = synth.make_x(cfg, li, device=DEV)
    wd = synth.make_w(cfg, li, device=DEV)
    dyd = synth.make_dy(cfg, li, device=DEV)
    ws = torch.empty(llmq.llmq_fp8_linear_workspace_bytes(M, N, K), dtype=torch.uint8, device=DEV)
    offs = llmq.llmq_fp8_linear_workspace_offsets(M, N, K)
    Y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    dX = torch.empty((M, K), dtype=torch.bfloat16, device=DEV)
    dW = torch.empty((N, K), dtype=torch.bfloat16, device=DEV)
    amax_y = torch.zeros(1, dtype=torch.float32, device=DEV)
    if jit:
        sx, sw, sd = (torch.full((1,), -1.0, dtype=torch.float32, device=DEV) for _ in range(3))
        llmq.llmq_fp8_linear_fwd(xd, wd, M, N, K, sx, sw, Y, amax_y, ws, llmq.JIT_X | llmq.JIT_W)
        llmq.llmq_fp8_linear_dgrad(dyd, None, M, N, K, sd, sw, fmt_dy, dX, None, ws, llmq.JIT_DY | llmq.REUSE_W)
    else:
        _, sx = gpu_amax(xd, 0)
        _, sw = gpu_amax(wd, 0)
        _, sd = gpu_amax(dyd, fmt_dy)
        llmq.llmq_fp8_linear_fwd(xd, wd, M, N, K, sx, sw, Y, amax_y, ws)
        llmq.llmq_fp8_linear_dgrad(dyd, None, M, N, K, sd, sw, fmt_dy, dX, None, ws, llmq.REUSE_W)
    llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, sd, sx, fmt_dy, dW, False, ws, llmq.REUSE_X | llmq.REUSE_DY)
    torch.cuda.synchronize()
    print("  gpu done; oracle quantize", flush=True)
    ox = oracle_quantized(xd, 0)
    ow = oracle_quantized(wd, 0)
    od = oracle_quantized(dyd, fmt_dy)
    assert [f32_bits(t) for t in (sx, sw, sd)] == [np_f32_bits(o[1]) for o in (ox, ow, od)]
    wsh = ws.cpu().numpy()
    for off, want in zip(offs, (ox[2], ox[3], ow[2], ow[3], od[2], od[3])):
        assert np.array_equal(wsh[off:off + want.size].reshape(want.shape), want)
    del wsh
    assert amax_y.item() == Y.float().abs().max().item()
    for name, out, (A, fa, sa), (B, fb, sb) in [
            ("fwd", Y, (ox[2], 0, ox[1]), (ow[2], 0, ow[1])),
            ("dgrad", dX, (od[2], fmt_dy, od[1]), (ow[3], 0, ow[1])),
            ("wgrad", dW, (od[3], fmt_dy, od[1]), (ox[3], 0, ox[1]))]:
        print("  oracle samples %s" % name, flush=True)
        rr, cc = _sample_positions(out.shape[0], out.shape[1], 4096, 17 + li)
        y, S = oracle.gemm_tn_sampled(A, fa, B, fb, sa, sb, rr, cc)
        got = out[torch.from_numpy(rr).to(DEV), torch.from_numpy(cc).to(DEV)].cpu().to(torch.float64).numpy()
        err = np.abs(got - y)
        assert np.all(err <= GEMM_TOL * S), (name, err.max(), (GEMM_TOL * S)[err.argmax()])
        assert np.isfinite(got).all() and np.abs(got).max() > 0


def test_all_tile_shapes_give_the_same_bytes_run_after_run():
    """Every wave-tile instantiation accumulates each output in the same order, so they must agree
    byte for byte, and every repetition with itself (more workgroups than CUs, few K steps: the
    situation in which a late direct-to-LDS zero fill once overwrote a staged output tile)."""
    import os
    R = C = 3072
    for T in (256, 384, 1152):
        A = _rand_codes((R, T), 0, 7 + T)
        B = _rand_codes((C, T), 0, 9 + T)
        Ad, Bd = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
        dsa, dsb = _scales(1.7, 0.3)
        ref = None
        try:
            for tile in ["4x4", "2x2", "4x3", "3x4", "3x3", "4x2", "2x4", "3x2", "2x3"]:
                os.environ["LLMQ_GEMM_TILE"] = tile
                for rep in range(3):
                    c = torch.full((R, C), float("nan"), dtype=torch.bfloat16, device=DEV)
                    llmq.llmq_fp8_gemm_tn(Ad, 0, Bd, 0, dsa, dsb, c, False, None)
                    if ref is None:
                        ref = c
                    else:
                        same = torch.equal(c.view(torch.int16), ref.view(torch.int16))
                        assert same, "tile %s repetition %d differs (T=%d)" % (tile, rep, T)
        finally:
            os.environ.pop("LLMQ_GEMM_TILE", None)
        rr, cc = _sample_positions(R, C, 512, 3)
        y, S = oracle.gemm_tn_sampled(A, 0, B, 0, 1.7, 0.3, rr, cc)
        got = ref[torch.from_numpy(rr).to(DEV), torch.from_numpy(cc).to(DEV)].cpu().to(torch.float64).numpy()
        assert np.all(np.abs(got - y) <= GEMM_TOL * S)


def test_tile_walk_and_touch_settings_do_not_change_any_byte(monkeypatch):
    """Band height of the tile walk, shares and distance of the L2 touch loads (tuning overrides) only move
    loads whose results are dropped and change which workgroup computes which tile: outputs and the fused absmax
    stay the same for every setting, on row-wise and T-major operands, with a ragged last band (9 tile rows)."""
    R, C, T = 9 * 256, 5 * 256, 896
    A = _rand_codes((R, T), 1, 31)
    B = _rand_codes((C, T), 0, 32)
    Ad, Bd = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    At, Bt = Ad.t().contiguous(), Bd.t().contiguous()
    dsa, dsb = _scales(1.3, 0.9)
    monkeypatch.setenv("LLMQ_GEMM_TILE", "4x4")

    def run(ta, tb):
        c = torch.full((R, C), float("nan"), dtype=torch.bfloat16, device=DEV)
        am = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
        llmq.llmq_fp8_gemm(At if ta else Ad, 1, ta, Bt if tb else Bd, 0, tb, dsa, dsb, c, False, am)
        return c, am

    ref, ref_am = run(False, False)
    y, S = oracle.gemm_tn(A, 1, B, 0, 1.3, 0.9)
    assert_gemm_close(ref, y, S, "default walk")
    for band, sa, sb, touch in [(1, 1, 1, 0), (2, 64, 64, 1), (8, 4, 8, 2), (64, 2, 3, 5), (3, 5, 7, 9)]:
        for k, v in (("LLMQ_GEMM_BAND", band), ("LLMQ_GEMM_SHARE_A", sa), ("LLMQ_GEMM_SHARE_B", sb), ("LLMQ_GEMM_TOUCH", touch)):
            monkeypatch.setenv(k, str(v))
        for ta, tb in ((False, False), (False, True), (True, True)):
            c, am = run(ta, tb)
            assert torch.equal(c.view(torch.int16), ref.view(torch.int16)), (band, sa, sb, touch, ta, tb)
            assert f32_bits(am) == f32_bits(ref_am)


@pytest.mark.parametrize("shape", [(256, 512, 1024), (272, 400, 528), (33, 17, 5), (4096, 1024, 768)])
@pytest.mark.parametrize("fmt_dy", [1, 0])
def test_just_in_time_scaling_inside_the_linear_calls(shape, fmt_dy):
    """LLMQ_JIT_*: the call finds the scale itself (first absmax stage + the quantize kernel finishing the
    reduction).  Scales, every workspace copy and every output must be the bytes of the explicit sequence
    llmq_amax -> call with the scale given; the scales are also checked against the oracle."""
    M, K, N = shape
    print("jit linear M=%d K=%d N=%d fmt_dy=%d" % (M, K, N, fmt_dy), flush=True)
    g = torch.Generator().manual_seed(M + 3 * K + 7 * N)
    x = torch.randn((M, K), generator=g).to(torch.bfloat16)
    w = (torch.randn((N, K), generator=g) * 0.02).to(torch.bfloat16)
    dy = (torch.randn((M, N), generator=g) * 1e-3).to(torch.bfloat16)
    xd, wd, dyd = x.to(DEV), w.to(DEV), dy.to(DEV)
    nbytes = llmq.llmq_fp8_linear_workspace_bytes(M, N, K)
    offs = llmq.llmq_fp8_linear_workspace_offsets(M, N, K)
    sizes = [M * K, M * K, N * K, N * K, M * N, M * N]

    def run(jit):
        ws = torch.full((nbytes,), 0x55, dtype=torch.uint8, device=DEV)          # scratch part starts as garbage
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
        dX = torch.empty((M, K), dtype=torch.bfloat16, device=DEV)
        dW = torch.empty((N, K), dtype=torch.bfloat16, device=DEV)
        ay = torch.zeros(1, device=DEV)
        adx = torch.zeros(1, device=DEV)
        if jit:
            sx, sw, sd = (torch.full((1,), -1.0, device=DEV) for _ in range(3))
            llmq.llmq_fp8_linear_fwd(xd, wd, M, N, K, sx, sw, Y, ay, ws, llmq.JIT_X | llmq.JIT_W)
            llmq.llmq_fp8_linear_dgrad(dyd, None, M, N, K, sd, sw, fmt_dy, dX, adx, ws, llmq.JIT_DY | llmq.REUSE_W)
            llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, sd, sx, fmt_dy, dW, False, ws, llmq.REUSE_X | llmq.REUSE_DY)
        else:
            _, sx = gpu_amax(xd, 0)
            _, sw = gpu_amax(wd, 0)
            _, sd = gpu_amax(dyd, fmt_dy)
            llmq.llmq_fp8_linear_fwd(xd, wd, M, N, K, sx, sw, Y, ay, ws)
            llmq.llmq_fp8_linear_dgrad(dyd, None, M, N, K, sd, sw, fmt_dy, dX, adx, ws, llmq.REUSE_W)
            llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, sd, sx, fmt_dy, dW, False, ws, llmq.REUSE_X | llmq.REUSE_DY)
        copies = [ws[o:o + n].clone() for o, n in zip(offs, sizes)]
        return (sx, sw, sd), copies, (Y, dX, dW), (ay, adx)

    s0, c0, o0, a0 = run(False)
    s1, c1, o1, a1 = run(True)
    assert [f32_bits(t) for t in s0] == [f32_bits(t) for t in s1]
    want = [oracle.scale(oracle.amax_bf16(synth.bf16_bits(t)), f) for t, f in ((x, 0), (w, 0), (dy, fmt_dy))]
    assert [f32_bits(t) for t in s1] == [np_f32_bits(v) for v in want]
    for a, b in zip(c0, c1):
        assert torch.equal(a, b)
    for a, b in zip(o0, o1):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert [f32_bits(t) for t in a0] == [f32_bits(t) for t in a1]
    # wgrad may also scale its own operands just in time (no forward or dgrad before it)
    ws = torch.full((nbytes,), 0xAA, dtype=torch.uint8, device=DEV)
    sd2, sx2 = torch.full((1,), -1.0, device=DEV), torch.full((1,), -1.0, device=DEV)
    dW2 = torch.empty((N, K), dtype=torch.bfloat16, device=DEV)
    llmq.llmq_fp8_linear_wgrad(dyd, xd, M, N, K, sd2, sx2, fmt_dy, dW2, False, ws, llmq.JIT_DY | llmq.JIT_X)
    assert f32_bits(sd2) == f32_bits(s0[2]) and f32_bits(sx2) == f32_bits(s0[0])
    assert torch.equal(dW2.view(torch.int16), o0[2].view(torch.int16))
    # an all-zero operand: scale 1, result zero
    z = torch.zeros_like(xd)
    sz, sw3 = torch.full((1,), -1.0, device=DEV), torch.full((1,), -1.0, device=DEV)
    Yz = torch.full((M, N), 3.0, dtype=torch.bfloat16, device=DEV)
    llmq.llmq_fp8_linear_fwd(z, wd, M, N, K, sz, sw3, Yz, None, ws, llmq.JIT_X | llmq.JIT_W)
    assert sz.item() == 1.0 and (Yz == 0).all()
    # flag combinations that make no sense are refused
    with pytest.raises(llmq.LlmqError) as e:
        llmq.llmq_fp8_linear_fwd(xd, wd, M, N, K, sz, sw3, Yz, None, ws, llmq.JIT_X | llmq.REUSE_X)
    assert e.value.status == -7
    with pytest.raises(llmq.LlmqError) as e:
        llmq.llmq_fp8_linear_fwd(xd, wd, M, N, K, sz, sw3, Yz, None, ws, llmq.JIT_DY)
    assert e.value.status == -7


def _block_step(cfg, states):
    for s in states:
        M, K, N = s["M"], s["K"], s["N"]
        llmq.llmq_amax(s["X"], 0, s["f"][0:1], s["f"][1:2], s["aws"])
        llmq.llmq_amax(s["W"], 0, s["f"][2:3], s["f"][3:4], s["aws"])
        llmq.llmq_fp8_linear_fwd(s["X"], s["W"], M, N, K, s["f"][1:2], s["f"][3:4], s["Y"], s["f"][6:7], s["ws"])
        llmq.llmq_amax(s["dY"], 1, s["f"][4:5], s["f"][5:6], s["aws"])
        llmq.llmq_fp8_linear_dgrad(s["dY"], None, M, N, K, s["f"][5:6], s["f"][3:4], 1, s["dX"], s["f"][7:8], s["ws"],
                                   llmq.REUSE_W)
        llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, s["f"][5:6], s["f"][1:2], 1, s["dW"], False, s["ws"],
                                   llmq.REUSE_X | llmq.REUSE_DY)


def test_whole_block_step_is_deterministic_and_replays_from_a_graph():
    """Config 2's whole step (12 absmax, 12 quantize, 12 GEMM launches): same bytes on every run
    (Section 3 "Reproducibility"), and the same bytes again when the step is captured in a HIP graph and
    replayed several times with eager work in between."""
    cfg = synth.CONFIGS[2]
    states = []
    for li, lin in enumerate(cfg.linears):
        M, K, N = cfg.M, lin.K, lin.N
        states.append(dict(M=M, K=K, N=N, X=synth.make_x(cfg, li, device=DEV), W=synth.make_w(cfg, li, device=DEV),
                           dY=synth.make_dy(cfg, li, device=DEV),
                           ws=torch.zeros(llmq.llmq_fp8_linear_workspace_bytes(M, N, K), dtype=torch.uint8, device=DEV),
                           aws=torch.empty(llmq.llmq_amax_workspace_bytes(), dtype=torch.uint8, device=DEV),
                           f=torch.zeros(8, dtype=torch.float32, device=DEV),
                           Y=torch.empty((M, N), dtype=torch.bfloat16, device=DEV),
                           dX=torch.empty((M, K), dtype=torch.bfloat16, device=DEV),
                           dW=torch.empty((N, K), dtype=torch.bfloat16, device=DEV)))

    def snapshot():
        torch.cuda.synchronize()
        return [s[k].clone() for s in states for k in ("Y", "dX", "dW", "f", "ws")]

    def scrub():
        for s in states:
            for k in ("Y", "dX", "dW", "f"):
                s[k].zero_()

    def same(a, b):
        return all(torch.equal(x.view(torch.uint8), y.view(torch.uint8)) for x, y in zip(a, b))

    _block_step(cfg, states)
    ref = snapshot()
    for rep in range(3):
        scrub()
        _block_step(cfg, states)
        assert same(ref, snapshot()), "eager run %d differs" % rep
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        _block_step(cfg, states)
    for rep in range(3):
        scrub()                                   # eager work and a synchronisation between the replays
        torch.cuda.synchronize()
        g.replay()
        assert same(ref, snapshot()), "graph replay %d differs" % rep
