"""Benchmark of the FP8 linear path on one MI355X.

A step is one pass of the whole path over one block's linears (QKV, attention-out, gate/up, down):
per linear  absmax+scale of X and W, quantize+transpose both, forward GEMM (with fused output absmax),
absmax+scale of dY, quantize+transpose, dgrad GEMM, wgrad GEMM, through the three linear calls with
just-in-time scaling.  Inputs are resident in HBM.

Prints ONE JSON line: whole-step TFLOP/s (6*M*K*N summed over the linears / step time), the roofline
of the dominant kernel (the FP8 MFMA GEMM, timed live with events on the launch stream) and the CPU
oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP8_TFLOPS = 5000.0      # MI355X dense FP8 MFMA, published
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense BF16 MFMA, published
PEAK_HBM_GBPS = 8000.0        # MI355X HBM3E, published
# L2 <-> fabric bytes per GEMM launch (fetched + written, averaged over the step's launches), from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script scaled by a plain 1 GiB copy
# (profiles/bench_config<N>_gemm_quantize_amax.md); None where not measured.  They include hits in the
# memory-side last-level cache: the 8 XCDs have private L2s and each re-reads the operands of its tiles.
MEASURED_GEMM_TRAFFIC_BYTES = {2: 221.5e6, 3: 940.1e6, 4: 1070.5e6, 5: 3660.1e6}
HEADLINE_CONFIG = 5           # the largest single-GPU configuration (32B-class block)
SIDE_CONFIGS = (3, 4)         # 7B- and 14B-class blocks: reported in the same line


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=20)
    p.add_argument("--warmup", type=int, default=5)
    p.add_argument("--config", type=int, default=0,
                   help="benchmark config index (2 = 3B-class block ... 5 = 32B-class); default: config 5 as the "
                        "headline with configs 3 and 4 (the other shapes the target is quoted on) as side entries")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--prequantized-w", action="store_true",
                   help="weights quantized once outside the timed region (reused across micro-steps)")
    p.add_argument("--whole-tiles", action="store_true",
                   help="linear calls without LLMQ_SHARE_TILES: every output tile is computed whole")
    p.add_argument("--plain-copies", action="store_true",
                   help="linear calls without LLMQ_SLAB_COPIES: transposed FP8 copies as plain transposed tensors")
    p.add_argument("--phase-stamps", action="store_true",
                   help="instead of the benchmark: cycle stamps of the phases of the GEMM tile kernel on two forward GEMMs")
    p.add_argument("--power-probe", action="store_true",
                   help="instead of the benchmark: one 8192^3 FP8 GEMM on operands of different bit content (zeros, one "
                        "constant, quantized Gaussian data, random codes) with the board power sampled from sysfs")
    return p.parse_args()


class LinearState:
    def __init__(self, cfg, li, dev):
        import torch
        from paper_2512_15306_amd import llmq, synth
        lin = cfg.linears[li]
        self.name, self.M, self.K, self.N = lin.name, cfg.M, lin.K, lin.N
        M, K, N = self.M, self.K, self.N
        self.X = synth.make_x(cfg, li, device=dev)
        self.W = synth.make_w(cfg, li, device=dev)
        self.dY = synth.make_dy(cfg, li, device=dev)
        self.ws = torch.empty(llmq.llmq_fp8_linear_workspace_bytes_shared(M, N, K), dtype=torch.uint8, device=dev)
        self.offs = llmq.llmq_fp8_linear_workspace_offsets(M, N, K)
        self.Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        self.dX = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
        self.dW = torch.empty((N, K), dtype=torch.bfloat16, device=dev)
        self.aws = torch.empty(llmq.llmq_amax_workspace_bytes(), dtype=torch.uint8, device=dev)
        self.f = torch.zeros(8, dtype=torch.float32, device=dev)   # amax/scale of X, W, dY; amax of Y, dX
        f = self.f
        self.ax, self.sx, self.aw, self.sw, self.ad, self.sd, self.ay, self.adx = (f[i:i + 1] for i in range(8))

    def view(self, which):
        M, K, N = self.M, self.K, self.N
        shape = {0: (M, K), 1: (K, M), 2: (N, K), 3: (K, N), 4: (M, N), 5: (N, M)}[which]
        o = self.offs[which]
        return self.ws[o:o + shape[0] * shape[1]].view(shape)


# Flags every linear call of the step carries unless a leg says otherwise (set in main from --whole-tiles).
DEFAULT_LINEAR_FLAGS = {"flags": 0}


def run_step(states, prequantized_w, producer_absmax=False, extra_flags=None):
    """Per linear: absmax + scale + quantize(+transpose) of X and W inside the forward call (just-in-time
    scaling: first absmax stage, then the quantize kernel finishes the reduction), forward GEMM, the same for
    dY inside the dgrad call, dgrad GEMM, wgrad GEMM on the copies already there.
    producer_absmax: the absmax passes over X and dY are left out, as when the producing kernel (RMSNorm,
    SwiGLU, the previous GEMM's epilogue) has already delivered them; the scales of the last full step are
    used.  Reported as a side figure only.
    extra_flags: LLMQ_NO_TRANSPOSE for the side figure without transposed copies; by default LLMQ_SHARE_TILES (the
    contractions may share a ragged last round of tiles among all compute units; --whole-tiles turns it off) and
    LLMQ_SLAB_COPIES (transposed copies stored in slabs of 128 contraction bytes; --plain-copies turns it off)."""
    from paper_2512_15306_amd import llmq
    if extra_flags is None:
        extra_flags = DEFAULT_LINEAR_FLAGS["flags"]
    for s in states:
        M, K, N = s.M, s.K, s.N
        fx = extra_flags | (0 if producer_absmax else llmq.JIT_X)
        fw = llmq.REUSE_W if prequantized_w else llmq.JIT_W
        llmq.llmq_fp8_linear_fwd(s.X, s.W, M, N, K, s.sx, s.sw, s.Y, s.ay, s.ws, fx | fw)
        fd = extra_flags | (0 if producer_absmax else llmq.JIT_DY)
        llmq.llmq_fp8_linear_dgrad(s.dY, None, M, N, K, s.sd, s.sw, llmq.E5M2, s.dX, s.adx, s.ws, llmq.REUSE_W | fd)
        llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, s.sd, s.sx, llmq.E5M2, s.dW, False, s.ws,
                                   extra_flags | llmq.REUSE_X | llmq.REUSE_DY)


def run_gemms_only(states, extra_flags=None, accumulate_dw=False):
    """The three GEMM launches of every linear on the operands the step left in the workspace, through
    the same entry points as the step (all REUSE flags set: nothing is quantized).  accumulate_dw: the weight
    gradients are added to dW in BF16 (one rounding), as on every micro-step of a gradient accumulation but
    the first."""
    from paper_2512_15306_amd import llmq
    if extra_flags is None:
        extra_flags = DEFAULT_LINEAR_FLAGS["flags"]
    for s in states:
        M, K, N = s.M, s.K, s.N
        llmq.llmq_fp8_linear_fwd(None, None, M, N, K, s.sx, s.sw, s.Y, None, s.ws, extra_flags | llmq.REUSE_X | llmq.REUSE_W)
        llmq.llmq_fp8_linear_dgrad(None, None, M, N, K, s.sd, s.sw, llmq.E5M2, s.dX, None, s.ws,
                                   extra_flags | llmq.REUSE_DY | llmq.REUSE_W)
        llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, s.sd, s.sx, llmq.E5M2, s.dW, accumulate_dw, s.ws,
                                   extra_flags | llmq.REUSE_X | llmq.REUSE_DY)


def quantizer():
    """The quantize call of the standalone legs: the transposed copy in the layout the step's linear calls use."""
    from paper_2512_15306_amd import llmq
    return llmq.llmq_quantize_fp8_slabs if DEFAULT_LINEAR_FLAGS["flags"] & llmq.SLAB_COPIES else llmq.llmq_quantize_fp8


def run_quant_only(states):
    from paper_2512_15306_amd import llmq
    quantize = quantizer()
    for s in states:
        llmq.llmq_amax(s.X, 0, s.ax, s.sx, s.aws)
        quantize(s.X, s.sx, 0, s.view(0), s.view(1))
        llmq.llmq_amax(s.W, 0, s.aw, s.sw, s.aws)
        quantize(s.W, s.sw, 0, s.view(2), s.view(3))
        llmq.llmq_amax(s.dY, 1, s.ad, s.sd, s.aws)
        quantize(s.dY, s.sd, 1, s.view(4), s.view(5))


def run_amax_only(states):
    from paper_2512_15306_amd import llmq
    for s in states:
        llmq.llmq_amax(s.X, 0, s.ax, s.sx, s.aws)
        llmq.llmq_amax(s.W, 0, s.aw, s.sw, s.aws)
        llmq.llmq_amax(s.dY, 1, s.ad, s.sd, s.aws)


def run_quantize_kernel_only(states):
    quantize = quantizer()
    for s in states:
        quantize(s.X, s.sx, 0, s.view(0), s.view(1))
        quantize(s.W, s.sw, 0, s.view(2), s.view(3))
        quantize(s.dY, s.sd, 1, s.view(4), s.view(5))


def run_quantize_row_major_only(states):
    from paper_2512_15306_amd import llmq
    for s in states:
        llmq.llmq_quantize_fp8(s.X, s.sx, 0, s.view(0), None)
        llmq.llmq_quantize_fp8(s.W, s.sw, 0, s.view(2), None)
        llmq.llmq_quantize_fp8(s.dY, s.sd, 1, s.view(4), None)


def timed(fn, reps):
    """Average milliseconds per call of fn over reps calls, by events on the current stream."""
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / reps


def measure_peaks(dev):
    """What this chip sustains: the GEMM's MFMA instruction from registers (constant and random operand
    bits) and a plain 1 GiB copy.  Reported next to the published peaks."""
    import torch
    from paper_2512_15306_amd import llmq
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    out = {}
    for name, rnd in (("mfma_fp8_const_bits_tflops", False), ("mfma_fp8_random_bits_tflops", True)):
        flops = llmq.llmq_calibrate_mfma(0, 0, rnd, 2000, sink)
        ms = timed(lambda: llmq.llmq_calibrate_mfma(0, 0, rnd, 20000, sink), 3)
        out[name] = round(flops * 10 / (ms * 1e-3) / 1e12, 1)
    src = torch.full((1 << 30,), 7, dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    llmq.llmq_calibrate_copy(src, dst)
    ms = timed(lambda: llmq.llmq_calibrate_copy(src, dst), 5)
    out["hbm_copy_gbps"] = round(2.0 * src.numel() / (ms * 1e-3) / 1e9, 1)
    return out


def measure_bf16_baseline(cfg, dev, reps):
    """The same three GEMMs per linear in BF16 (no quantization): what a BF16 run of the block spends on its
    linears.  The kernel wants both operands contraction-contiguous, so the transposed copies a BF16
    framework would not need (it would use other GEMM layouts) are made outside the timed region."""
    import torch
    from paper_2512_15306_amd import llmq, synth
    ops = []
    for li, lin in enumerate(cfg.linears):
        X, W, dY = synth.make_x(cfg, li, device=dev), synth.make_w(cfg, li, device=dev), synth.make_dy(cfg, li, device=dev)
        Xt, Wt, dYt = X.t().contiguous(), W.t().contiguous(), dY.t().contiguous()
        M, K, N = cfg.M, lin.K, lin.N
        Y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        dX = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
        dW = torch.empty((N, K), dtype=torch.bfloat16, device=dev)
        ops += [(X, W, Y), (dY, Wt, dX), (dYt, Xt, dW)]

    def run():
        for a, b, c in ops:
            llmq.llmq_bf16_gemm_tn(a, b, c)
    run()
    ms = timed(run, reps)
    return ms


def measure_swiglu(cfg, dev, reps):
    """The block's SwiGLU with its fused outputs (next to the linears, not part of the step's FLOP count):
    forward writing h + absmax, recompute mode writing FP8 bytes (both layouts; the transposed copy plain or in
    slabs of 128 contraction bytes) instead of h, backward writing dGU + absmax.  GB/s on algorithmic bytes: 6, 6 and 10 per element of h."""
    import torch
    from paper_2512_15306_amd import llmq, synth
    M, I = synth.swiglu_dims(cfg)
    gu, dh = synth.make_gu(cfg, device=dev), synth.make_dh(cfg, device=dev)
    h = torch.empty((M, I), dtype=torch.bfloat16, device=dev)
    dgu = torch.empty((M, 2 * I), dtype=torch.bfloat16, device=dev)
    q = torch.empty((M, I), dtype=torch.uint8, device=dev)
    qt = torch.empty((I, M), dtype=torch.uint8, device=dev)
    f = torch.zeros(4, dtype=torch.float32, device=dev)
    ws = torch.empty(llmq.llmq_swiglu_workspace_bytes(M, I), dtype=torch.uint8, device=dev)
    aws = torch.empty(llmq.llmq_amax_workspace_bytes(), dtype=torch.uint8, device=dev)
    n = float(M) * I
    legs = {
        "fwd_h_absmax": (6.0, lambda: llmq.llmq_swiglu_fwd(gu, h, llmq.E4M3, f[0:1], f[1:2], ws)),
        "fwd_fp8_both_layouts": (6.0, lambda: llmq.llmq_swiglu_fwd_fp8(gu, f[1:2], llmq.E4M3, q, qt, None)),
        "fwd_fp8_slab_copy": (6.0, lambda: llmq.llmq_swiglu_fwd_fp8_slabs(gu, f[1:2], llmq.E4M3, q, qt, None)),
        "bwd_dgu_absmax": (10.0, lambda: llmq.llmq_swiglu_bwd(dh, gu, dgu, llmq.E5M2, f[2:3], f[3:4], ws)),
        "separate_absmax_of_h": (2.0, lambda: llmq.llmq_amax(h, llmq.E4M3, f[0:1], f[1:2], aws)),
        "separate_quantize_of_h": (4.0, lambda: llmq.llmq_quantize_fp8(h, f[1:2], llmq.E4M3, q, qt)),
    }
    out = {"M": M, "I": I}
    for name, (bpe, fn) in legs.items():
        fn()
        ms = timed(fn, reps)
        out[name] = {"ms": round(ms, 4), "gbps": round(bpe * n / (ms * 1e-3) / 1e9, 1),
                     "pct_hbm_peak": round(100.0 * bpe * n / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 2)}
    return out


def measure_rmsnorm(cfg, dev, reps):
    """RMSNorm + residual addition in front of the block's first linear: forward (res', y, rstd, absmax:
    4 B read + 4 B written per element) and the recompute path (stored stream + statistics -> FP8 in both
    layouts: 2 B read + 2 B written)."""
    import torch
    from paper_2512_15306_amd import llmq, synth
    res, x, w = synth.make_norm_inputs(cfg, device=dev)
    M, C = res.shape
    res_out, y = torch.empty_like(res), torch.empty_like(res)
    rstd = torch.empty(M, dtype=torch.float32, device=dev)
    q = torch.empty((M, C), dtype=torch.uint8, device=dev)
    qt = torch.empty((C, M), dtype=torch.uint8, device=dev)
    f = torch.ones(2, dtype=torch.float32, device=dev)
    ws = torch.empty(llmq.llmq_rmsnorm_workspace_bytes(M), dtype=torch.uint8, device=dev)
    n = float(M) * C
    legs = {
        "fwd_add_norm_absmax": (8.0, lambda: llmq.llmq_rmsnorm_fwd(res, x, w, 1e-6, res_out, y, rstd, llmq.E4M3, f[0:1], f[1:2], ws)),
        "recompute_fp8_both_layouts": (4.0, lambda: llmq.llmq_rmsnorm_apply_fp8(res_out, w, rstd, f[1:2], llmq.E4M3, q, qt, None)),
        "recompute_fp8_slab_copy": (4.0, lambda: llmq.llmq_rmsnorm_apply_fp8_slabs(res_out, w, rstd, f[1:2], llmq.E4M3, q, qt, None)),
    }
    out = {"M": M, "C": C}
    for name, (bpe, fn) in legs.items():
        fn()
        ms = timed(fn, reps)
        out[name] = {"ms": round(ms, 4), "gbps": round(bpe * n / (ms * 1e-3) / 1e9, 1),
                     "pct_hbm_peak": round(100.0 * bpe * n / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 2)}
    return out


def power_probe(dev):
    """The same 8192 x 8192 x 8192 contraction on operands that differ only in their bits, each run for about a
    second while a thread samples the board power (hwmon power1_input, microwatts).  Shows what bounds the GEMM
    on real data: the power cap, not the kernel."""
    import glob
    import threading
    import torch
    from paper_2512_15306_amd import llmq
    hw = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*"))

    def read(name):
        for h in hw:
            try:
                return float(open(os.path.join(h, name)).read())
            except (OSError, ValueError):
                pass
        return None

    class Poller(threading.Thread):
        def __init__(self):
            super().__init__(daemon=True)
            self.stop, self.samples = False, []

        def run(self):
            while not self.stop:
                v = read("power1_input")
                if v is None:
                    v = read("power1_average")
                if v is not None:
                    self.samples.append(v / 1e6)
                time.sleep(0.02)

    n = 8192
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    aws = torch.empty(llmq.llmq_amax_workspace_bytes(), dtype=torch.uint8, device=dev)
    f = torch.zeros(2, dtype=torch.float32, device=dev)

    def quantized(x):                       # through the library: absmax scale, E4M3 codes
        q = torch.empty((n, n), dtype=torch.uint8, device=dev)
        llmq.llmq_amax(x, llmq.E4M3, f[0:1], f[1:2], aws)
        llmq.llmq_quantize_fp8(x, f[1:2], llmq.E4M3, q, None)
        return q

    def operand(kind, seed):
        g.manual_seed(seed)
        if kind == "zeros":
            return torch.zeros((n, n), dtype=torch.uint8, device=dev)
        if kind == "one_constant":
            return torch.full((n, n), 0x38, dtype=torch.uint8, device=dev)
        if kind == "quantized_gaussian":
            return quantized(torch.randn((n, n), generator=g, device=dev).to(torch.bfloat16))
        if kind == "quantized_gaussian_outlier_channels":      # 0.5 % of the columns x 50, as config 3's activations
            x = torch.randn((n, n), generator=g, device=dev)
            x[:, torch.randperm(n, generator=torch.Generator().manual_seed(seed))[:41].to(dev)] *= 50.0
            return quantized(x.to(torch.bfloat16))
        # random finite codes: random sign and mantissa, exponent field 3 .. 10
        e = torch.randint(3, 11, (n, n), generator=g, device=dev, dtype=torch.int32)
        m = torch.randint(0, 8, (n, n), generator=g, device=dev, dtype=torch.int32)
        sg = torch.randint(0, 2, (n, n), generator=g, device=dev, dtype=torch.int32)
        return ((sg << 7) | (e << 3) | m).to(torch.uint8)

    one = torch.ones(1, dtype=torch.float32, device=dev)
    c = torch.empty((n, n), dtype=torch.bfloat16, device=dev)
    out = {"what": "8192^3 E4M3 x E4M3 GEMM (llmq_fp8_gemm_tn), about one second per operand pattern, board power "
                   "from hwmon power1_input sampled every 20 ms (second half of the run averaged)",
           "power_cap_watts": (read("power1_cap") or 0) / 1e6, "patterns": {}}
    for kind in ("zeros", "one_constant", "quantized_gaussian_outlier_channels", "quantized_gaussian", "random_codes"):
        A, B = operand(kind, 11), operand(kind, 12)
        fn = lambda: llmq.llmq_fp8_gemm_tn(A, 0, B, 0, one, one, c, False, None)
        ms1 = timed(fn, 20)
        reps = max(50, int(1000.0 / ms1))
        p = Poller()
        p.start()
        ms = timed(fn, reps)
        p.stop = True
        p.join()
        half = p.samples[len(p.samples) // 2:]
        out["patterns"][kind] = {"tflops": round(2.0 * n ** 3 / (ms * 1e-3) / 1e12, 1), "ms": round(ms, 4),
                                 "watts": round(sum(half) / len(half), 1) if half else None, "samples": len(half)}
        del A, B
        time.sleep(0.5)
    return out


def phase_stamps(dev):
    """Cycle stamps of the phases of the 256 x 256 tile kernel (llmq_calibrate_gemm_phases) on the forward GEMM of
    config 3's gate/up projection (19 rounds of tiles, 28 K steps) and of config 2's attention-out projection (one
    round, 24 K steps), operands quantized from the configs' tensors; averages over the workgroups, for the fused
    absmax as the library computes it and for the maxNum form it replaced."""
    import torch
    from paper_2512_15306_amd import llmq, synth
    out = {}
    aws = torch.empty(llmq.llmq_amax_workspace_bytes(), dtype=torch.uint8, device=dev)
    for ci, li in ((3, 2), (2, 1)):
        cfg = synth.CONFIGS[ci]
        lin = cfg.linears[li]
        f = torch.zeros(5, dtype=torch.float32, device=dev)
        ops = []
        for t, sl in ((synth.make_x(cfg, li, device=dev), 0), (synth.make_w(cfg, li, device=dev), 2)):
            q = torch.empty(t.shape, dtype=torch.uint8, device=dev)
            llmq.llmq_amax(t, llmq.E4M3, f[sl:sl + 1], f[sl + 1:sl + 2], aws)
            llmq.llmq_quantize_fp8(t, f[sl + 1:sl + 2], llmq.E4M3, q, None)
            ops.append(q)
        c = torch.empty((cfg.M, lin.N), dtype=torch.bfloat16, device=dev)
        entry = {"R": cfg.M, "C": lin.N, "T": lin.K, "tiles": (cfg.M // 256) * (lin.N // 256), "k_steps": lin.K // 128}
        for name, ieee in (("ieee_maximum", True), ("maxnum", False)):
            for _ in range(3):
                st = llmq.llmq_calibrate_gemm_phases(ops[0], ops[1], f[1:2], f[3:4], c, f[4:5], ieee)
            torch.cuda.synchronize()
            s = st.cpu().double()
            s = s[s[:, 0] > 0]
            cyc = lambda a, b: float((s[:, b] - s[:, a]).mean())
            ns = lambda a, b: float((s[:, 8 + b] - s[:, 8 + a]).mean()) * 10.0          # 100 MHz stamps
            entry[name] = {
                "workgroups": int(s.shape[0]),
                "prologue_cycles": round(cyc(0, 1)), "k_loop_cycles": round(cyc(1, 2)),
                "k_loop_cycles_per_step": round(cyc(1, 2) / (lin.K // 128), 1),
                "epilogue_to_last_store_issued_cycles": round(cyc(2, 4)), "absmax_tail_cycles": round(cyc(4, 5)),
                "epilogue_until_stores_complete_cycles": round(cyc(2, 3)), "whole_tile_cycles": round(cyc(0, 3)),
                "whole_tile_ns": round(ns(0, 3)), "clock_ghz": round(cyc(0, 3) / ns(0, 3), 3)}
        out["config %d %s forward" % (ci, lin.name)] = entry
    return out


def cpu_baseline(cfg):
    """The oracle as it stands on a bounded sample: the largest linear of the block restricted to the
    first rows of the token dimension, whole path (3 absmax, 3 quantize+transpose, 3 fp64 GEMMs)."""
    import oracle
    from paper_2512_15306_amd import synth
    li = max(range(len(cfg.linears)), key=lambda i: cfg.linears[i].K * cfg.linears[i].N)   # the largest linear
    lin = cfg.linears[li]
    # size the sample for roughly 15 s on this host: time a 32-row slab of the forward GEMM first
    import numpy as np
    probe = np.zeros((32, lin.K), np.uint8)
    wprobe = np.zeros((lin.N, lin.K), np.uint8)
    oracle.gemm_tn(probe[:1], 0, wprobe[:8], 0, 1.0, 1.0)      # load the library
    t0 = time.perf_counter()
    oracle.gemm_tn(probe, 0, wprobe, 0, 1.0, 1.0)
    per_row = (time.perf_counter() - t0) / 32 * 3.0             # three GEMMs per token row
    Ms = int(min(cfg.M, max(64, 15.0 / max(per_row, 1e-9))))
    Ms -= Ms % 16
    del probe, wprobe
    x = synth.bf16_bits(synth.make_x(cfg, li, M=Ms))
    w = synth.bf16_bits(synth.make_w(cfg, li))
    dy = synth.bf16_bits(synth.make_dy(cfg, li, M=Ms))
    oracle.amax_bf16(x[:8])            # load the library outside the timed region
    t0 = time.perf_counter()
    sx = oracle.scale(oracle.amax_bf16(x), 0)
    sw = oracle.scale(oracle.amax_bf16(w), 0)
    sd = oracle.scale(oracle.amax_bf16(dy), 1)
    xq, xqt = oracle.quantize(x, sx, 0)
    wq, wqt = oracle.quantize(w, sw, 0)
    dq, dqt = oracle.quantize(dy, sd, 1)
    oracle.gemm_tn(xq, 0, wq, 0, sx, sw)
    oracle.gemm_tn(dq, 1, wqt, 0, sd, sw)
    oracle.gemm_tn(dqt, 1, xqt, 0, sd, sx)
    dt = time.perf_counter() - t0
    flops = 6.0 * Ms * lin.K * lin.N
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "seconds": round(dt, 2),
            "sample": "config %d '%s' linear (K=%d, N=%d) on the first %d of %d tokens: absmax, "
                      "quantize+transpose and fp64 fwd/dgrad/wgrad" % (cfg.index, lin.name, lin.K, lin.N, Ms, cfg.M)}


def measure_config(cfg, args, dev, full):
    """One configuration: the timed step (args.warmup untimed, args.steps timed), then the GEMM launches alone
    (the roofline of the dominant kernel) and the absmax / quantize legs on the same operands.  full: also
    the side figures (no transposed copies, producer-fused absmax).  Returns a dict of raw figures."""
    import torch
    from paper_2512_15306_amd import llmq, synth
    states = [LinearState(cfg, li, dev) for li in range(len(cfg.linears))]
    if args.prequantized_w:
        for s in states:
            llmq.llmq_amax(s.W, llmq.E4M3, s.aw, s.sw, s.aws)
            quantizer()(s.W, s.sw, llmq.E4M3, s.view(2), s.view(3))
    for _ in range(args.warmup):
        run_step(states, args.prequantized_w)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms_step = timed(lambda: run_step(states, args.prequantized_w), args.steps)
    wall = (time.perf_counter() - t0) * 1e3 / args.steps
    flops = float(synth.linear_flops(cfg))
    # dominant kernel: the FP8 GEMM (three launches per linear), timed alone on the same operands
    reps = max(3, min(args.steps, 20))
    r = {"cfg": cfg, "flops": flops, "ms_step": ms_step, "wall": wall, "reps": reps, "n_gemm": 3 * len(states),
         "elements": float(synth.quantize_elements(cfg))}
    r["ms_gemm"] = timed(lambda: run_gemms_only(states), reps)
    r["ms_quant"] = timed(lambda: run_quant_only(states), reps)
    r["ms_amax"] = timed(lambda: run_amax_only(states), reps)
    r["ms_qk"] = timed(lambda: run_quantize_kernel_only(states), reps)
    if full:
        r["ms_fused"] = timed(lambda: run_step(states, args.prequantized_w, producer_absmax=True), reps)
        r["ms_qrow"] = timed(lambda: run_quantize_row_major_only(states), reps)
        for s in states:
            s.dW.zero_()                               # sums of a few dozen equal gradients stay finite in BF16
        r["ms_gemm_acc"] = timed(lambda: run_gemms_only(states, accumulate_dw=True), reps)
        # the same step on row-major FP8 copies only (the backward GEMMs read them T-major): a side figure
        run_step(states, args.prequantized_w, extra_flags=llmq.NO_TRANSPOSE)       # first use loads those kernels
        r["ms_nt"] = timed(lambda: run_step(states, args.prequantized_w, extra_flags=llmq.NO_TRANSPOSE), reps)
        r["ms_nt_gemm"] = timed(lambda: run_gemms_only(states, llmq.NO_TRANSPOSE), reps)
        r["ms_nt_fused"] = timed(lambda: run_step(states, args.prequantized_w, producer_absmax=True, extra_flags=llmq.NO_TRANSPOSE), reps)
    del states
    torch.cuda.empty_cache()
    return r


def workload_name(cfg, prequantized_w):
    return ("config %d: %s, M=%d tokens, linears %s; absmax + quantize(+transpose) of X, W, dY "
            "(e4m3, e4m3, e5m2) and fwd+dgrad+wgrad per linear%s" % (
                cfg.index, cfg.name, cfg.M, ", ".join("%s %dx%d" % (l.name, l.K, l.N) for l in cfg.linears),
                "; W pre-quantized" if prequantized_w else ""))


def roofline_of(r):
    """One "launch" is one contraction (a linear call with all REUSE flags): one kernel launch, or three where the
    last round of tiles is shared out (pieces, their sums, the whole rounds; LLMQ_SHARE_TILES)."""
    gemm_tflops = r["flops"] / (r["ms_gemm"] * 1e-3) / 1e12
    return {"kernel": "gemm_tile_kernel", "bound": "mfma", "achieved": round(gemm_tflops, 2),
            "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s", "frac": round(gemm_tflops / PEAK_FP8_TFLOPS, 4),
            "traffic": MEASURED_GEMM_TRAFFIC_BYTES.get(r["cfg"].index), "launches_per_step": r["n_gemm"],
            "avg_launch_ms": round(r["ms_gemm"] / r["n_gemm"], 5), "flops_per_launch": r["flops"] / r["n_gemm"]}


def rate_fields(r):
    """Whole-step and per-leg rates of one configuration (the fields the headline and the side entries share)."""
    flops, n = r["flops"], r["elements"]
    value = flops / (r["ms_step"] * 1e-3) / 1e12
    gemm_tflops = flops / (r["ms_gemm"] * 1e-3) / 1e12
    gbps = lambda bpe, ms: bpe * n / (ms * 1e-3) / 1e9
    return {
        "ms_per_step": round(r["ms_step"], 4),
        "step_tflops": round(value, 2), "pct_fp8_peak": round(100.0 * value / PEAK_FP8_TFLOPS, 2),
        "gemm_only_tflops": round(gemm_tflops, 2),
        "gemm_only_pct_fp8_peak": round(100.0 * gemm_tflops / PEAK_FP8_TFLOPS, 2),
        # absmax reads 2 B, quantize reads 2 B and writes 1 + 1 B per element
        "quantize_gbps": round(gbps(6.0, r["ms_quant"]), 1),
        "quantize_pct_hbm_peak": round(100.0 * gbps(6.0, r["ms_quant"]) / PEAK_HBM_GBPS, 2),
        "absmax_only_gbps": round(gbps(2.0, r["ms_amax"]), 1),
        "absmax_only_pct_hbm_peak": round(100.0 * gbps(2.0, r["ms_amax"]) / PEAK_HBM_GBPS, 2),
        "quantize_kernel_only_gbps": round(gbps(4.0, r["ms_qk"]), 1),
        "quantize_kernel_only_pct_hbm_peak": round(100.0 * gbps(4.0, r["ms_qk"]) / PEAK_HBM_GBPS, 2),
    }


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not "
              "supported, use --gpus 1" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2512_15306_amd import llmq, synth
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    llmq.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.phase_stamps:
        print(json.dumps({"phase_stamps": phase_stamps(dev)}))
        return
    if args.power_probe:
        print(json.dumps({"power_probe": power_probe(dev)}))
        return
    DEFAULT_LINEAR_FLAGS["flags"] = (0 if args.whole_tiles else llmq.SHARE_TILES) | (0 if args.plain_copies else llmq.SLAB_COPIES)
    cfg = synth.CONFIGS[args.config or HEADLINE_CONFIG]
    peaks = measure_peaks(dev)
    r = measure_config(cfg, args, dev, full=True)
    flops, ms_step, ms_gemm, reps = r["flops"], r["ms_step"], r["ms_gemm"], r["reps"]
    n = r["elements"]
    rates = rate_fields(r)
    gemm_tflops = rates["gemm_only_tflops"]
    out = {
        "metric": "FP8 linear fwd+bwd TFLOP/s and % dense-FP8 MFMA peak; quantize GB/s",
        "value": rates["step_tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rates["ms_per_step"], "wall_ms_per_step": round(r["wall"], 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "fp8", "data": "synthetic",
        "config": {"workload": workload_name(cfg, args.prequantized_w)},
        "linear_flags": "LLMQ_JIT_* (scales found inside the calls)" + ("" if args.whole_tiles else " | LLMQ_SHARE_TILES") + ("" if args.plain_copies else " | LLMQ_SLAB_COPIES"),
    }
    out.update({k: v for k, v in rates.items() if k not in ("ms_per_step", "step_tflops")})
    out.update({
        "quantize_row_major_only_gbps": round(3.0 * n / (r["ms_qrow"] * 1e-3) / 1e9, 1),
        "quantize_row_major_only_pct_hbm_peak": round(100.0 * 3.0 * n / (r["ms_qrow"] * 1e-3) / 1e9 / PEAK_HBM_GBPS, 2),
        "step_tflops_with_producer_fused_absmax": round(flops / (r["ms_fused"] * 1e-3) / 1e12, 2),
        "step_tflops_without_transposed_copies": round(flops / (r["ms_nt"] * 1e-3) / 1e12, 2),
        "gemm_only_tflops_without_transposed_copies": round(flops / (r["ms_nt_gemm"] * 1e-3) / 1e12, 2),
        "gemm_only_tflops_with_bf16_accumulation_of_dw": round(flops / (r["ms_gemm_acc"] * 1e-3) / 1e12, 2),
        "step_tflops_without_transposed_copies_with_producer_fused_absmax": round(flops / (r["ms_nt_fused"] * 1e-3) / 1e12, 2),
        "measured_peaks": peaks,
        "gemm_only_pct_measured_random_bits_peak": round(100.0 * gemm_tflops / peaks["mfma_fp8_random_bits_tflops"], 2),
        "quantize_pct_measured_copy": round(100.0 * rates["quantize_gbps"] / peaks["hbm_copy_gbps"], 2),
        "roofline": roofline_of(r),
    })
    if not args.config:
        # the other shapes the target is quoted on, each timed the same way (same warm-up and step counts)
        sides = {}
        for ci in SIDE_CONFIGS:
            rs = measure_config(synth.CONFIGS[ci], args, dev, full=False)
            e = {"workload": workload_name(synth.CONFIGS[ci], args.prequantized_w)}
            e.update(rate_fields(rs))
            e["roofline"] = roofline_of(rs)
            sides["config %d" % ci] = e
        out["side_configs"] = sides
    ms_bf16 = measure_bf16_baseline(cfg, dev, reps)
    torch.cuda.empty_cache()
    bf16_tflops = flops / (ms_bf16 * 1e-3) / 1e12
    out["bf16_baseline"] = {
        "what": "fwd+dgrad+wgrad GEMMs of the same linears on BF16 operands (v_mfma_f32_16x16x32_bf16, same tile "
                "kernel), no quantization, pre-transposed operands",
        "ms_per_step": round(ms_bf16, 4), "tflops": round(bf16_tflops, 2),
        "pct_bf16_peak": round(100.0 * bf16_tflops / PEAK_BF16_TFLOPS, 2),
        "fp8_gemm_only_speedup": round(ms_bf16 / ms_gemm, 3),
        "fp8_whole_step_speedup": round(ms_bf16 / ms_step, 3)}
    out["swiglu"] = measure_swiglu(cfg, dev, reps)
    out["rmsnorm"] = measure_rmsnorm(cfg, dev, reps)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
