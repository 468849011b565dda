"""Quantization error of the output gradients in E4M3 and in E5M2 (paper Section 5, Scenario 1: the
all-E4M3 configuration tracked the BF16 run more closely than E5M2 gradients did).

For every linear of benchmark configs 2-5 the script draws the config's dY tensor (seeded, the same bytes the
GPU tests and bench.py use), quantizes it with the oracle to both formats with tensor-level absmax scaling,
decodes the codes again and reports, per tensor and format:
  rel_rms   sqrt( sum (dec(q)/s - x)^2 / sum x^2 ), in binary64
  flushed   share of non-zero elements whose code is +-0
  subnorm   share of elements that land on a subnormal code (reduced precision)
  at_fmax   number of elements on the largest code (the absmax element(s); nothing else may clip)
It calls nothing but oracle/ and the input generator.  Usage:
    python oracle/dy_format_error.py [--configs 2 3 4 5] [--out tests/golden/dy_format_error.txt]
tests/test_oracle_dy_formats.py recomputes rows of the stored table.
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2512_15306_amd import synth  # noqa: E402

MBITS = {oracle.E4M3: 3, oracle.E5M2: 2}
NAMES = {oracle.E4M3: "e4m3", oracle.E5M2: "e5m2"}


def tensor_stats(dy_bits: np.ndarray, fmt: int, rows_per_chunk: int = 512):
    """dy_bits: [M, N] uint16 BF16 patterns.  Returns (scale, rel_rms, flushed, subnorm, at_fmax)."""
    amax = oracle.amax_bf16(dy_bits)
    s = oracle.scale(amax, fmt)
    table = oracle.decode_table(fmt)
    max_code = 0x7E if fmt == oracle.E4M3 else 0x7B
    first_normal = 1 << MBITS[fmt]                     # magnitude codes below it are zero or subnormal
    num = den = 0.0
    flushed = nonzero = subnorm = at_fmax = 0
    for r0 in range(0, dy_bits.shape[0], rows_per_chunk):
        xb = dy_bits[r0:r0 + rows_per_chunk]
        q, _ = oracle.quantize(xb, s, fmt, transpose=False)
        x = (xb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        d = table[q] / float(s)
        num += float(np.sum((d - x) ** 2))
        den += float(np.sum(x * x))
        mag = q & 0x7F
        nz = x != 0.0
        nonzero += int(nz.sum())
        flushed += int((nz & (mag == 0)).sum())
        subnorm += int(((mag > 0) & (mag < first_normal)).sum())
        at_fmax += int((mag == max_code).sum())
    n = dy_bits.size
    return float(s), (num / den) ** 0.5, flushed / max(nonzero, 1), subnorm / n, at_fmax


def row_text(ci, lin, M, fmt, st):
    return "%d %-8s %6d %6d %s %.9e %.6e %.6e %.6e %d" % ((ci, lin.name, M, lin.N, NAMES[fmt]) + st)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", type=int, nargs="*", default=[2, 3, 4, 5])
    ap.add_argument("--out", default=os.path.join(ROOT, "tests", "golden", "dy_format_error.txt"))
    args = ap.parse_args()
    lines = ["# written by oracle/dy_format_error.py (oracle only); paper Section 5, Scenario 1",
             "# config linear M N format scale rel_rms flushed_share subnormal_share at_fmax"]
    for ci in args.configs:
        cfg = synth.CONFIGS[ci]
        for li, lin in enumerate(cfg.linears):
            dy = synth.bf16_bits(synth.make_dy(cfg, li)).reshape(cfg.M, lin.N)
            for fmt in (oracle.E4M3, oracle.E5M2):
                line = row_text(ci, lin, cfg.M, fmt, tensor_stats(dy, fmt))
                print(line, flush=True)
                lines.append(line)
            del dy
    with open(args.out, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", args.out)


if __name__ == "__main__":
    main()
