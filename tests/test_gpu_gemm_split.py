"""GPU parity of the deterministic split of the contraction (ragged last round of tiles shared among all CUs;
paper Section 3 "Reproducibility": partial results in an intermediate buffer, added in a fixed order by a second
step).  Small problems are pushed onto that path with the tuning overrides LLMQ_GEMM_SLOTS (workgroups the planner
believes the chip holds at once) and LLMQ_GEMM_SPLIT."""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_15306_amd import llmq, synth
from gpu_common import DEV, GEMM_TOL, f32_bits, gpu_amax, bf16_to_f64, assert_gemm_close
from test_gpu_gemm import _rand_codes, _scales, _sample_positions

pytestmark = pytest.mark.gpu


def _run(A, fa, ta, B, fb, tb, sa, sb, scratch_mb=64, accumulate=False, c_init=None, want_amax=True):
    Ad, Bd = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    if ta:
        Ad = Ad.t().contiguous()
    if tb:
        Bd = Bd.t().contiguous()
    dsa, dsb = _scales(sa, sb)
    c = torch.full((A.shape[0], B.shape[0]), float("nan"), dtype=torch.bfloat16, device=DEV) if c_init is None else c_init.clone()
    am = torch.full((1,), -1.0, dtype=torch.float32, device=DEV) if want_amax else None
    scratch = torch.full((scratch_mb << 20,), 0xFF, dtype=torch.uint8, device=DEV) if scratch_mb else None   # NaN patterns on entry
    llmq.llmq_fp8_gemm_with_scratch(Ad, fa, ta, Bd, fb, tb, dsa, dsb, c, accumulate, am, scratch)
    return c, am


@pytest.mark.parametrize("split", ["a2", "a3", "a9", "1"])
@pytest.mark.parametrize("T", [1152, 640])
@pytest.mark.parametrize("ta,tb", [(False, False)])
def test_shared_tiles_match_the_oracle_and_repeat_bit_for_bit(split, T, ta, tb, monkeypatch):
    """15 tiles of 256 x 256 with the planner told the chip holds 8 workgroups: 8 tiles are computed whole, 7 are
    cut into 2, 3 or 9 pieces (one K step each at T = 1152) or as the planner likes; odd and even piece lengths."""
    R, C = 3 * 256, 5 * 256
    monkeypatch.setenv("LLMQ_GEMM_TILE", "4x4")
    monkeypatch.setenv("LLMQ_GEMM_SLOTS", "8")
    monkeypatch.setenv("LLMQ_GEMM_SPLIT", split)
    print("split=%s T=%d ta=%d tb=%d" % (split, T, ta, tb), flush=True)
    A = _rand_codes((R, T), 1, 5 + T)
    B = _rand_codes((C, T), 0, 6 + T)
    c, am = _run(A, 1, ta, B, 0, tb, 1.9, 0.7)
    y, S = oracle.gemm_tn(A, 1, B, 0, 1.9, 0.7)
    assert_gemm_close(c, y, S, "split " + split)
    a2, _ = gpu_amax(c.reshape(-1), 0, want_scale=False)
    assert f32_bits(am) == f32_bits(a2)
    for rep in range(2):                        # same bytes every time (fixed order of the additions)
        c2, am2 = _run(A, 1, ta, B, 0, tb, 1.9, 0.7)
        assert torch.equal(c2.view(torch.int16), c.view(torch.int16)) and f32_bits(am2) == f32_bits(am)
    # the sharing really happened: without scratch every tile is computed whole, which groups the additions
    # differently, so at least the two results must both be within tolerance, and pieces of one K step each
    # (a9 at T = 1152) can differ from the whole-tile result only by rounding
    c0, _ = _run(A, 1, ta, B, 0, tb, 1.9, 0.7, scratch_mb=0)
    assert_gemm_close(c0, y, S, "whole")
    diff = (bf16_to_f64(c0) - bf16_to_f64(c)) != 0
    assert diff.mean() < 0.05


def test_split_with_bf16_accumulation(monkeypatch):
    monkeypatch.setenv("LLMQ_GEMM_SLOTS", "8")
    monkeypatch.setenv("LLMQ_GEMM_SPLIT", "a3")
    for tile, (R, C) in (("4x4", (4 * 256, 3 * 256)), ("4x4", (2 * 256, 7 * 256))):
        monkeypatch.setenv("LLMQ_GEMM_TILE", tile)
        T = 896
        A = _rand_codes((R, T), 0, 15)
        B = _rand_codes((C, T), 0, 16)
        g = torch.Generator().manual_seed(4)
        c0 = (torch.randn((R, C), generator=g) * 40).to(torch.bfloat16).to(DEV)
        c, _ = _run(A, 0, False, B, 0, False, 2.0, 0.5, accumulate=True, c_init=c0, want_amax=False)
        y, S = oracle.gemm_tn(A, 0, B, 0, 2.0, 0.5)
        want = bf16_to_f64(c0) + y
        assert np.all(np.abs(bf16_to_f64(c) - want) <= GEMM_TOL * S + 2.0 ** -8 * np.abs(want)), tile
        c1, am = _run(A, 0, False, B, 0, False, 2.0, 0.5)
        assert_gemm_close(c1, y, S, "split " + tile)
        assert am.item() == c1.float().abs().max().item()


def test_scratch_is_ignored_for_t_major_operands(monkeypatch):
    """Sharing exists for contraction-contiguous operands only: with a T-major operand the call computes every tile
    whole, scratch or not, and gives the bytes of llmq_fp8_gemm."""
    monkeypatch.setenv("LLMQ_GEMM_TILE", "4x4")
    monkeypatch.setenv("LLMQ_GEMM_SLOTS", "8")
    monkeypatch.setenv("LLMQ_GEMM_SPLIT", "a3")
    R, C, T = 3 * 256, 5 * 256, 768
    A = _rand_codes((R, T), 1, 51)
    B = _rand_codes((C, T), 0, 52)
    for ta, tb in ((False, True), (True, True), (True, False)):
        c1, am1 = _run(A, 1, ta, B, 0, tb, 1.9, 0.7)
        c0, am0 = _run(A, 1, ta, B, 0, tb, 1.9, 0.7, scratch_mb=0)
        assert torch.equal(c1.view(torch.int16), c0.view(torch.int16)) and f32_bits(am1) == f32_bits(am0)


def test_integer_inputs_stay_exact_when_tiles_are_shared(monkeypatch):
    """Small integers: every partial sum is exact in binary32, so shared and whole tiles must agree bit for bit
    and equal the integer matmul rounded once to BF16."""
    monkeypatch.setenv("LLMQ_GEMM_TILE", "4x4")
    monkeypatch.setenv("LLMQ_GEMM_SLOTS", "8")
    R, C, T = 3 * 256, 3 * 256, 768
    rng = np.random.default_rng(3)
    vals = np.array([0x00, 0x38, 0xB8, 0x40, 0xC0], dtype=np.uint8)          # 0, 1, -1, 2, -2 in E4M3
    A, B = vals[rng.integers(0, 5, (R, T))], vals[rng.integers(0, 5, (C, T))]
    dec = oracle.decode_table(0)
    want = torch.from_numpy(dec[A] @ dec[B].T).to(torch.bfloat16).to(torch.float64).numpy()
    g = torch.Generator().manual_seed(8)
    c0 = (torch.round(torch.randn((R, C), generator=g) * 160) / 4).to(torch.bfloat16)        # multiples of 1/4
    exact = bf16_to_f64(c0) + dec[A] @ dec[B].T                 # fits binary32 exactly: one rounding is left
    want_acc = torch.from_numpy(exact).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    for split in ("0", "a2", "a6"):
        monkeypatch.setenv("LLMQ_GEMM_SPLIT", split)
        c, _ = _run(A, 0, False, B, 0, False, 1.0, 1.0)
        assert np.array_equal(bf16_to_f64(c), want), split
        # the sums launch of the shared tiles with BF16 accumulation: old value + exact sum, rounded once
        c, am = _run(A, 0, False, B, 0, False, 1.0, 1.0, accumulate=True, c_init=c0.to(DEV))
        assert np.array_equal(bf16_to_f64(c), want_acc), split
        assert am.item() == np.abs(want_acc).max(), split


@pytest.mark.parametrize("cfg_i,li,which", [(4, 2, "dgrad"), (5, 0, "wgrad"), (5, 3, "wgrad")])
def test_full_size_gemms_the_planner_shares(cfg_i, li, which):
    """Shapes of the benchmark configurations that the library shares out by itself (long contractions whose
    tile count leaves a ragged last round: 640 tiles = 2 rounds + 128, 560 = 2 + 48, 2160 = 8 + 112): with scratch
    of the size the library asks for, sampled outputs against the oracle, equality run to run, and the fused
    absmax against the stored tensor."""
    cfg = synth.CONFIGS[cfg_i]
    lin = cfg.linears[li]
    M, K, N = cfg.M, lin.K, lin.N
    R, C, T = {"fwd": (M, N, K), "dgrad": (M, K, N), "wgrad": (N, K, M)}[which]
    need = llmq.llmq_fp8_gemm_scratch_bytes(R, C, T)
    print("config %d %s %s R=%d C=%d T=%d scratch %d MB" % (cfg_i, lin.name, which, R, C, T, need >> 20), flush=True)
    assert need > 0, "the planner no longer shares this shape: pick another one for the test"
    A = _rand_codes((R, T), 1, 21 + li)
    B = _rand_codes((C, T), 0, 22 + li)
    Ad, Bd = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    dsa, dsb = _scales(3.0, 0.25)
    scratch = torch.full((need,), 0xFF, dtype=torch.uint8, device=DEV)
    outs = []
    for rep in range(2):
        c = torch.full((R, C), float("nan"), dtype=torch.bfloat16, device=DEV)
        am = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
        llmq.llmq_fp8_gemm_with_scratch(Ad, 1, False, Bd, 0, False, dsa, dsb, c, False, am, scratch)
        outs.append((c, am))
    assert torch.equal(outs[0][0].view(torch.int16), outs[1][0].view(torch.int16))
    c, am = outs[0]
    assert am.item() == c.float().abs().max().item()
    rr, cc = _sample_positions(R, C, 4096, 5)
    # every tile of the last tile row and column is sampled too: that is where the shared tiles sit
    extra_r = np.concatenate([np.full(C // 64, R - 1 - 256 * (i % 2)) for i in range(2)])
    extra_c = np.concatenate([np.arange(0, C, 64) for _ in range(2)])
    rr, cc = np.concatenate([rr, extra_r]), np.concatenate([cc, extra_c])
    y, S = oracle.gemm_tn_sampled(A, 1, B, 0, 3.0, 0.25, rr, cc)
    got = c[torch.from_numpy(rr).to(DEV), torch.from_numpy(cc).to(DEV)].cpu().to(torch.float64).numpy()
    assert np.all(np.abs(got - y) <= GEMM_TOL * S)
    assert not torch.isnan(c).any()


@pytest.mark.parametrize("cfg_i,li", [(5, 0), (4, 2), (3, 1)])
def test_linear_calls_that_may_share_tiles(cfg_i, li):
    """LLMQ_SHARE_TILES on the three linear calls, as bench.py's step carries it: config 5's qkv projection (its
    weight gradient shares tiles), config 4's gate/up projection (its input gradient does) and config 3's
    attention-out projection (nothing is shared).  Outputs of contractions that share nothing are the bytes of the
    calls without the flag; the others are checked against the oracle on sampled outputs, with the last tile row
    and column among them, and must come out the same bytes when run again."""
    cfg = synth.CONFIGS[cfg_i]
    lin = cfg.linears[li]
    M, K, N = cfg.M, lin.K, lin.N
    print("config %d %s M=%d K=%d N=%d" % (cfg_i, lin.name, M, K, N), flush=True)
    X, W, dY = synth.make_x(cfg, li, device=DEV), synth.make_w(cfg, li, device=DEV), synth.make_dy(cfg, li, device=DEV)
    ws = torch.full((llmq.llmq_fp8_linear_workspace_bytes_shared(M, N, K),), 0xFF, dtype=torch.uint8, device=DEV)
    sx, sw, sd = (torch.zeros(1, dtype=torch.float32, device=DEV) for _ in range(3))

    def run(flags):
        Y = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
        dX = torch.full((M, K), float("nan"), dtype=torch.bfloat16, device=DEV)
        dW = torch.full((N, K), float("nan"), dtype=torch.bfloat16, device=DEV)
        adx = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
        llmq.llmq_fp8_linear_fwd(X, W, M, N, K, sx, sw, Y, None, ws, flags | llmq.JIT_X | llmq.JIT_W)
        llmq.llmq_fp8_linear_dgrad(dY, None, M, N, K, sd, sw, llmq.E5M2, dX, adx, ws, flags | llmq.JIT_DY | llmq.REUSE_W)
        llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, sd, sx, llmq.E5M2, dW, False, ws, flags | llmq.REUSE_X | llmq.REUSE_DY)
        torch.cuda.synchronize()
        return Y, dX, dW, adx

    whole = run(0)
    shared = run(llmq.SHARE_TILES)
    again = run(llmq.SHARE_TILES)
    offs = llmq.llmq_fp8_linear_workspace_offsets(M, N, K)
    copy = lambda i, r, c: ws[offs[i]:offs[i] + r * c].view(r, c).cpu().numpy()
    operands = {"fwd": (copy(0, M, K), 0, copy(2, N, K), 0, sx, sw, (M, N, K)),
                "dgrad": (copy(4, M, N), 1, copy(3, K, N), 0, sd, sw, (M, K, N)),
                "wgrad": (copy(5, N, M), 1, copy(1, K, M), 0, sd, sx, (N, K, M))}
    any_shared = False
    for k, which in enumerate(("fwd", "dgrad", "wgrad")):
        A, fa, B, fb, sa, sb, (R, C, T) = operands[which]
        assert torch.equal(shared[k].view(torch.int16), again[k].view(torch.int16)), which
        assert not torch.isnan(shared[k]).any(), which
        if llmq.llmq_fp8_gemm_scratch_bytes(R, C, T) == 0:
            assert torch.equal(shared[k].view(torch.int16), whole[k].view(torch.int16)), which
            continue
        any_shared = True
        rr, cc = _sample_positions(R, C, 2048, 7 + k)
        extra_r = np.concatenate([np.full(C // 64, R - 1 - 256 * (i % 2)) for i in range(2)])
        extra_c = np.concatenate([np.arange(0, C, 64) for _ in range(2)])
        rr, cc = np.concatenate([rr, extra_r]), np.concatenate([cc, extra_c])
        y, S = oracle.gemm_tn_sampled(A, fa, B, fb, sa.item(), sb.item(), rr, cc)
        got = shared[k][torch.from_numpy(rr).to(DEV), torch.from_numpy(cc).to(DEV)].cpu().to(torch.float64).numpy()
        assert np.all(np.abs(got - y) <= GEMM_TOL * S), which
    assert any_shared == (cfg_i != 3)
    assert shared[3].item() == shared[1].float().abs().max().item()
