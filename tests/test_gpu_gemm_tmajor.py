"""GPU parity of the FP8 contraction on T-major operands (no transposed copies) and of the linear calls
under LLMQ_NO_TRANSPOSE: against the fp64 oracle, and bit for bit against the contraction on explicit
transposes, which sums the same products in the same accumulator positions."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_15306_amd import llmq, synth
from gpu_common import DEV, GEMM_TOL, f32_bits, gpu_amax, oracle_quantized, assert_gemm_close
from test_gpu_gemm import _rand_codes, _scales, _sample_positions, _linear_case

pytestmark = pytest.mark.gpu

LAYOUTS = [(False, True), (True, True), (True, False)]


def _run(A, fa, ta, B, fb, tb, sa, sb, accumulate=False, c_init=None, want_amax=False):
    """A [R,T], B [C,T] as numpy codes; a T-major operand is handed over as its transpose, made contiguous."""
    Ad = torch.from_numpy(np.ascontiguousarray(A.T) if ta else A).to(DEV)
    Bd = torch.from_numpy(np.ascontiguousarray(B.T) if tb else B).to(DEV)
    dsa, dsb = _scales(sa, sb)
    c = torch.full((A.shape[0], B.shape[0]), float("nan"), dtype=torch.bfloat16, device=DEV) if c_init is None else c_init.clone()
    am = torch.full((1,), -1.0, dtype=torch.float32, device=DEV) if want_amax else None
    llmq.llmq_fp8_gemm(Ad, fa, ta, Bd, fb, tb, dsa, dsb, c, accumulate, am)
    return c, am


def _run_tn(A, fa, B, fb, sa, sb, accumulate=False, c_init=None):
    dsa, dsb = _scales(sa, sb)
    c = torch.full((A.shape[0], B.shape[0]), float("nan"), dtype=torch.bfloat16, device=DEV) if c_init is None else c_init.clone()
    llmq.llmq_fp8_gemm_tn(torch.from_numpy(A).to(DEV), fa, torch.from_numpy(B).to(DEV), fb, dsa, dsb, c, accumulate, None)
    return c


# generic path: odd shapes, ragged T; tuned path: multiples of the tiles (odd and even numbers of K steps)
SHAPES = [(1, 1, 1), (5, 3, 7), (33, 17, 130), (100, 136, 72), (256, 256, 128), (256, 512, 384), (512, 256, 640),
          (768, 1024, 512), (384, 384, 256)]


@pytest.mark.parametrize("R,C,T", SHAPES)
@pytest.mark.parametrize("ta,tb", LAYOUTS)
@pytest.mark.parametrize("fa,fb", [(0, 0), (1, 0), (0, 1)])
def test_t_major_operands_within_tolerance(R, C, T, ta, tb, fa, fb):
    print("gemm R=%d C=%d T=%d ta=%d tb=%d fa=%d fb=%d" % (R, C, T, ta, tb, fa, fb), flush=True)
    A = _rand_codes((R, T), fa, 11 * R + T + fa)
    B = _rand_codes((C, T), fb, 13 * C + T + fb + 1)
    sa, sb = 3.7, 0.61
    c, am = _run(A, fa, ta, B, fb, tb, sa, sb, want_amax=True)
    y, S = oracle.gemm_tn(A, fa, B, fb, sa, sb)
    assert_gemm_close(c, y, S, "gemm")
    assert am.item() == c.float().abs().max().item()
    a2, _ = gpu_amax(c.reshape(-1), 0, want_scale=False)
    assert f32_bits(am) == f32_bits(a2)
    # The contraction on explicit transposes gives the same bytes where both run the same kind of kernel
    # (a T-major E5M2 B takes the generic kernel, whose MFMA shape sums in another order than the tuned tiles).
    if fb == 0 or R % 128 or C % 128 or T % 128:
        assert torch.equal(_run_tn(A, fa, B, fb, sa, sb).view(torch.int16), c.view(torch.int16))


def test_both_layouts_false_is_the_tn_call():
    A = _rand_codes((256, 384), 1, 3)
    B = _rand_codes((512, 384), 0, 4)
    c, _ = _run(A, 1, False, B, 0, False, 1.5, 0.75)
    assert torch.equal(_run_tn(A, 1, B, 0, 1.5, 0.75).view(torch.int16), c.view(torch.int16))


@pytest.mark.parametrize("tile", ["4x4", "4x3", "4x2", "3x4", "3x3", "3x2", "2x4", "2x3", "2x2"])
@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_every_tuned_tile_shape_with_t_major_operands(tile, ta, tb, monkeypatch):
    """Each wave tile of the tuned kernel in each layout, on 2 x 3 workgroup tiles with an odd number of K
    steps and on a longer contraction with an even number; plain and accumulating epilogue."""
    ni, nj = int(tile[0]), int(tile[2])
    R, C = 2 * 64 * ni, 3 * 64 * nj
    monkeypatch.setenv("LLMQ_GEMM_TILE", tile)
    for T, fa in ((640, 1), (1024, 0)):
        print("tile %s ta=%d tb=%d R=%d C=%d T=%d" % (tile, ta, tb, R, C, T), flush=True)
        A = _rand_codes((R, T), fa, 41 + ni + T)
        B = _rand_codes((C, T), 0, 43 + nj + T)
        c, am = _run(A, fa, ta, B, 0, tb, 1.9, 0.7, want_amax=True)
        y, S = oracle.gemm_tn(A, fa, B, 0, 1.9, 0.7)
        assert_gemm_close(c, y, S, "tile " + tile)
        assert am.item() == c.float().abs().max().item()
        assert torch.equal(_run_tn(A, fa, B, 0, 1.9, 0.7).view(torch.int16), c.view(torch.int16))
        g = torch.Generator().manual_seed(5)
        c0 = (torch.randn((R, C), generator=g) * 20).to(torch.bfloat16).to(DEV)
        acc, _ = _run(A, fa, ta, B, 0, tb, 1.9, 0.7, accumulate=True, c_init=c0)
        want = _run_tn(A, fa, B, 0, 1.9, 0.7, accumulate=True, c_init=c0)
        assert torch.equal(want.view(torch.int16), acc.view(torch.int16))
        got = acc.double().cpu().numpy()
        ref = c0.double().cpu().numpy() + y
        assert np.all(np.abs(got - ref) <= GEMM_TOL * S + 2.0 ** -8 * np.abs(ref))


def test_operand_position_is_not_mixed_up():
    """One nonzero code per operand: the product must land at exactly one output, for every layout."""
    R, C, T = 256, 384, 256
    for (r, ka), (cc, kb) in (((3, 5), (7, 5)), ((200, 131), (300, 131)), ((255, 255), (383, 255)), ((17, 64), (90, 65))):
        A = np.zeros((R, T), np.uint8); B = np.zeros((C, T), np.uint8)
        A[r, ka] = 0x38      # 1.0 in E4M3
        B[cc, kb] = 0x40     # 2.0
        for ta, tb in LAYOUTS:
            c, _ = _run(A, 0, ta, B, 0, tb, 1.0, 1.0)
            got = c.float().cpu().numpy()
            want = np.zeros((R, C), np.float32)
            if ka == kb:
                want[r, cc] = 2.0
            assert np.array_equal(got, want), (r, ka, cc, kb, ta, tb)


@pytest.mark.parametrize("shape", synth.small_cases())
@pytest.mark.parametrize("fmt_dy", [1, 0])
def test_linear_calls_without_transposed_copies(shape, fmt_dy):
    """LLMQ_NO_TRANSPOSE: same Y, dX, dW bytes as the calls with transposed copies, the row-major copies are the
    oracle's, the transposed sections of the workspace stay untouched."""
    M, K, N = shape
    print("linear M=%d K=%d N=%d fmt_dy=%d" % (M, K, N, fmt_dy), flush=True)
    g = torch.Generator().manual_seed(M * 7 + K * 3 + N)
    x = torch.randn((M, K), generator=g).to(torch.bfloat16)
    w = (torch.randn((N, K), generator=g) * 0.02).to(torch.bfloat16)
    dy = (torch.randn((M, N), generator=g) * 1e-3).to(torch.bfloat16)
    _, sx, xq, xqt = oracle_quantized(x, 0)
    _, sw, wq, wqt = oracle_quantized(w, 0)
    _, sd, dq, dqt = oracle_quantized(dy, fmt_dy)
    xd, wd, dyd = x.to(DEV), w.to(DEV), dy.to(DEV)
    nbytes = llmq.llmq_fp8_linear_workspace_bytes(M, N, K)
    offs = llmq.llmq_fp8_linear_workspace_offsets(M, N, K)
    compact = llmq.llmq_fp8_linear_workspace_bytes_no_transpose(M, N, K)
    assert compact <= min(offs[1], offs[3], offs[5])
    outs = {}
    for flag in (0, llmq.NO_TRANSPOSE):
        full = torch.full((nbytes,), 0x55, dtype=torch.uint8, device=DEV)
        ws = full[:compact] if flag else full       # the bytes behind a compact workspace must stay untouched
        gsx = torch.zeros(1, dtype=torch.float32, device=DEV)
        gsw, gsd = torch.zeros_like(gsx), torch.zeros_like(gsx)
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
        dX = torch.empty((M, K), dtype=torch.bfloat16, device=DEV)
        dW = torch.zeros((N, K), dtype=torch.bfloat16, device=DEV)
        amax_y = torch.zeros(1, dtype=torch.float32, device=DEV)
        amax_dx = torch.zeros(1, dtype=torch.float32, device=DEV)
        llmq.llmq_fp8_linear_fwd(xd, wd, M, N, K, gsx, gsw, Y, amax_y, ws, flag | llmq.JIT_X | llmq.JIT_W)
        llmq.llmq_fp8_linear_dgrad(dyd, None, M, N, K, gsd, gsw, fmt_dy, dX, amax_dx, ws, flag | llmq.REUSE_W | llmq.JIT_DY)
        llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, gsd, gsx, fmt_dy, dW, True, ws, flag | llmq.REUSE_X | llmq.REUSE_DY)
        outs[flag] = (Y, dX, dW, amax_y.item(), amax_dx.item(), full.cpu().numpy())
    for a, b in zip(outs[0][:3], outs[llmq.NO_TRANSPOSE][:3]):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert outs[0][3:5] == outs[llmq.NO_TRANSPOSE][3:5]
    wsh = outs[llmq.NO_TRANSPOSE][5]
    assert (wsh[compact:] == 0x55).all()
    for i, want in enumerate((xq, xqt, wq, wqt, dq, dqt)):
        got = wsh[offs[i]:offs[i] + want.size]
        if i % 2 == 0:
            assert np.array_equal(got.reshape(want.shape), want)
        else:
            assert (got == 0x55).all()
    Y, dX, dW = outs[llmq.NO_TRANSPOSE][:3]
    y, S = oracle.gemm_tn(xq, 0, wq, 0, sx, sw)
    assert_gemm_close(Y, y, S, "fwd")
    y, S = oracle.gemm_tn(dq, fmt_dy, wqt, 0, sd, sw)
    assert_gemm_close(dX, y, S, "dgrad")
    y, S = oracle.gemm_tn(dqt, fmt_dy, xqt, 0, sd, sx)
    assert_gemm_close(dW, y, S, "wgrad")
    # the backward calls quantize for themselves when nothing is reused
    ws2 = torch.full((nbytes,), 0x33, dtype=torch.uint8, device=DEV)
    dX2 = torch.empty_like(dX)
    dW2 = torch.zeros_like(dW)
    gsx, gsw, gsd = (torch.tensor([v], dtype=torch.float32, device=DEV) for v in (sx, sw, sd))
    llmq.llmq_fp8_linear_dgrad(dyd, wd, M, N, K, gsd, gsw, fmt_dy, dX2, None, ws2, llmq.NO_TRANSPOSE)
    llmq.llmq_fp8_linear_wgrad(dyd, xd, M, N, K, gsd, gsx, fmt_dy, dW2, True, ws2, llmq.NO_TRANSPOSE)
    assert torch.equal(dX2.view(torch.int16), dX.view(torch.int16))
    assert torch.equal(dW2.view(torch.int16), dW.view(torch.int16))


@pytest.mark.parametrize("cfg_i,li", [(2, 0), (3, 2), (5, 1), (5, 3)])
def test_full_size_backward_without_transposed_copies(cfg_i, li):
    """Benchmark shapes: dgrad and wgrad on the row-major copies give the bytes of the calls on transposed
    copies, and sampled outputs agree with full-length dot products of the oracle."""
    cfg = synth.CONFIGS[cfg_i]
    lin = cfg.linears[li]
    M, K, N = cfg.M, lin.K, lin.N
    print("full-size config %d %s M=%d K=%d N=%d" % (cfg_i, lin.name, M, K, N), flush=True)
    xd = synth.make_x(cfg, li, device=DEV)
    wd = synth.make_w(cfg, li, device=DEV)
    dyd = synth.make_dy(cfg, li, device=DEV)
    _, sx = gpu_amax(xd, 0)
    _, sw = gpu_amax(wd, 0)
    _, sd = gpu_amax(dyd, 1)
    ws = torch.empty(llmq.llmq_fp8_linear_workspace_bytes(M, N, K), dtype=torch.uint8, device=DEV)
    res = {}
    for flag in (0, llmq.NO_TRANSPOSE):
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
        dX = torch.empty((M, K), dtype=torch.bfloat16, device=DEV)
        dW = torch.empty((N, K), dtype=torch.bfloat16, device=DEV)
        llmq.llmq_fp8_linear_fwd(xd, wd, M, N, K, sx, sw, Y, None, ws, flag)
        llmq.llmq_fp8_linear_dgrad(dyd, None, M, N, K, sd, sw, 1, dX, None, ws, flag | llmq.REUSE_W)
        llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, sd, sx, 1, dW, False, ws, flag | llmq.REUSE_X | llmq.REUSE_DY)
        torch.cuda.synchronize()
        res[flag] = (Y, dX, dW)
    for a, b in zip(res[0], res[llmq.NO_TRANSPOSE]):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    print("  gpu done; oracle quantize", flush=True)
    ox = oracle_quantized(xd, 0)
    ow = oracle_quantized(wd, 0)
    od = oracle_quantized(dyd, 1)
    _, dX, dW = res[llmq.NO_TRANSPOSE]
    for name, out, (A, fa, sa), (B, fb, sb) in [
            ("dgrad", dX, (od[2], 1, od[1]), (ow[3], 0, ow[1])),
            ("wgrad", dW, (od[3], 1, od[1]), (ox[3], 0, ox[1]))]:
        print("  oracle samples %s" % name, flush=True)
        rr, cc = _sample_positions(out.shape[0], out.shape[1], 2048, 23 + li)
        y, S = oracle.gemm_tn_sampled(A, fa, B, fb, sa, sb, rr, cc)
        got = out[torch.from_numpy(rr).to(DEV), torch.from_numpy(cc).to(DEV)].cpu().to(torch.float64).numpy()
        err = np.abs(got - y)
        assert np.all(err <= GEMM_TOL * S), (name, err.max())
        assert np.isfinite(got).all() and np.abs(got).max() > 0


@pytest.mark.parametrize("ta,tb", LAYOUTS)
def test_request_of_the_next_tiles_slabs_with_t_major_operands(ta, tb, monkeypatch):
    """272 tiles of 256 x 256 on 256 CUs with the successor's first slabs requested by every workgroup (forced
    through the tuning override; by default only long GEMMs do it): the loads must not change any byte."""
    R, C, T = 17 * 256, 16 * 256, 512
    A = _rand_codes((R, T), 1, 71)
    B = _rand_codes((C, T), 0, 72)
    monkeypatch.setenv("LLMQ_GEMM_TILE", "4x4")
    monkeypatch.setenv("LLMQ_GEMM_TOUCH_NEXT", "1")
    c, am = _run(A, 1, ta, B, 0, tb, 2.5, 0.5, want_amax=True)
    monkeypatch.setenv("LLMQ_GEMM_TOUCH_NEXT", "0")
    c0, _ = _run(A, 1, ta, B, 0, tb, 2.5, 0.5)
    assert torch.equal(c.view(torch.int16), c0.view(torch.int16))
    assert torch.equal(_run_tn(A, 1, B, 0, 2.5, 0.5).view(torch.int16), c.view(torch.int16))
    assert am.item() == c.float().abs().max().item()
    rr, cc = _sample_positions(R, C, 1024, 5)
    y, S = oracle.gemm_tn_sampled(A, 1, B, 0, 2.5, 0.5, rr, cc)
    got = c[torch.from_numpy(rr).to(DEV), torch.from_numpy(cc).to(DEV)].cpu().to(torch.float64).numpy()
    assert np.all(np.abs(got - y) <= GEMM_TOL * S)


def test_degenerate_scales_and_all_zero_operands_with_t_major_operands():
    """An all-zero operand with the largest finite scale (a tiny absmax gives it), and a scale product that leaves the normal range
    (second copy of the epilogue), in the T-major instantiations."""
    R, C, T = 256, 256, 256
    A = _rand_codes((R, T), 0, 81)
    Z = np.zeros((C, T), np.uint8)
    for ta, tb in LAYOUTS:
        c, am = _run(A, 0, ta, Z, 0, tb, 3.0, 3.4028234e38, want_amax=True)
        assert (c.view(torch.int16) & 0x7FFF).max().item() == 0 and am.item() == 0.0
        B = _rand_codes((C, T), 0, 82)
        big = 2.0 ** 65                  # 1 / (sA sB) = 2^-130 is below the normal range: two multiplies
        c, _ = _run(A, 0, ta, B, 0, tb, big, big)
        want = _run_tn(A, 0, B, 0, big, big)
        assert torch.equal(want.view(torch.int16), c.view(torch.int16))
        assert c.float().abs().max().item() > 0
        y, S = oracle.gemm_tn(A, 0, B, 0, big, big)
        assert_gemm_close(c, y, S, "tiny")


def test_step_without_transposed_copies_replays_from_a_graph():
    """The benchmark's side-figure step on config 2 (just-in-time scaling, row-major FP8 copies only, backward
    GEMMs on T-major operands, compact workspaces): the same bytes run after run, from a captured HIP graph
    replayed with eager work in between, and the same outputs as the step with transposed copies."""
    cfg = synth.CONFIGS[2]
    states = []
    for li, lin in enumerate(cfg.linears):
        M, K, N = cfg.M, lin.K, lin.N
        states.append(dict(M=M, K=K, N=N, X=synth.make_x(cfg, li, device=DEV), W=synth.make_w(cfg, li, device=DEV),
                           dY=synth.make_dy(cfg, li, device=DEV),
                           ws=torch.zeros(llmq.llmq_fp8_linear_workspace_bytes(M, N, K), dtype=torch.uint8, device=DEV),
                           f=torch.zeros(8, dtype=torch.float32, device=DEV),
                           Y=torch.empty((M, N), dtype=torch.bfloat16, device=DEV),
                           dX=torch.empty((M, K), dtype=torch.bfloat16, device=DEV),
                           dW=torch.empty((N, K), dtype=torch.bfloat16, device=DEV)))

    def step(flag):
        for s in states:
            M, K, N, f = s["M"], s["K"], s["N"], s["f"]
            ws = s["ws"][:llmq.llmq_fp8_linear_workspace_bytes_no_transpose(M, N, K)] if flag else s["ws"]
            llmq.llmq_fp8_linear_fwd(s["X"], s["W"], M, N, K, f[1:2], f[3:4], s["Y"], f[6:7], ws, flag | llmq.JIT_X | llmq.JIT_W)
            llmq.llmq_fp8_linear_dgrad(s["dY"], None, M, N, K, f[5:6], f[3:4], 1, s["dX"], f[7:8], ws, flag | llmq.REUSE_W | llmq.JIT_DY)
            llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, f[5:6], f[1:2], 1, s["dW"], False, ws, flag | llmq.REUSE_X | llmq.REUSE_DY)

    def snapshot(keys=("Y", "dX", "dW", "f")):
        torch.cuda.synchronize()
        return [s[k].clone() for s in states for k in keys]

    def scrub():
        for s in states:
            for k in ("Y", "dX", "dW", "f"):
                s[k].zero_()

    def same(a, b):
        return all(torch.equal(x.view(torch.uint8), y.view(torch.uint8)) for x, y in zip(a, b))

    step(0)
    with_copies = snapshot()
    scrub()
    step(llmq.NO_TRANSPOSE)
    ref = snapshot()
    assert same(with_copies, ref)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(llmq.NO_TRANSPOSE)
    for rep in range(3):
        scrub()
        torch.cuda.synchronize()
        g.replay()
        assert same(ref, snapshot()), "graph replay %d differs" % rep
