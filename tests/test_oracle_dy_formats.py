"""E4M3 against E5M2 for the output gradients (paper Section 5, Scenario 1): the stored table
tests/golden/dy_format_error.txt (written by oracle/dy_format_error.py from the oracle alone) is recomputed
for two tensors, and its content is checked against what the formats' arithmetic fixes."""
import importlib.util
import os

import numpy as np

import oracle
from paper_2512_15306_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TABLE = os.path.join(ROOT, "tests", "golden", "dy_format_error.txt")


def _script():
    spec = importlib.util.spec_from_file_location("dy_format_error", os.path.join(ROOT, "oracle", "dy_format_error.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _rows():
    out = []
    for line in open(TABLE):
        if line.startswith("#") or not line.strip():
            continue
        c, name, M, N, fmt, s, rms, flushed, sub, fmax = line.split()
        out.append(dict(config=int(c), linear=name, M=int(M), N=int(N), fmt=fmt, scale=float(s), rel_rms=float(rms),
                        flushed=float(flushed), subnorm=float(sub), at_fmax=int(fmax)))
    return out


def test_table_covers_every_linear_of_configs_2_to_5_in_both_formats():
    rows = _rows()
    want = {(ci, l.name, f) for ci in (2, 3, 4, 5) for l in synth.CONFIGS[ci].linears for f in ("e4m3", "e5m2")}
    assert {(r["config"], r["linear"], r["fmt"]) for r in rows} == want


def test_stored_rows_are_what_the_oracle_gives():
    mod = _script()
    rows = {(r["config"], r["linear"], r["fmt"]): r for r in _rows()}
    cfg = synth.CONFIGS[2]
    for li in (1, 3):                                       # o and down of config 2: 12.6 M elements each
        lin = cfg.linears[li]
        dy = synth.bf16_bits(synth.make_dy(cfg, li)).reshape(cfg.M, lin.N)
        for fmt, name in ((oracle.E4M3, "e4m3"), (oracle.E5M2, "e5m2")):
            s, rms, flushed, sub, fmax = mod.tensor_stats(dy, fmt)
            r = rows[(2, lin.name, name)]
            assert np.isclose(s, r["scale"], rtol=1e-9) and np.isclose(rms, r["rel_rms"], rtol=1e-6)
            assert np.isclose(flushed, r["flushed"], rtol=1e-6, atol=1e-12) and np.isclose(sub, r["subnorm"], rtol=1e-6, atol=1e-12)
            assert fmax == r["at_fmax"]


def test_error_levels_follow_from_the_mantissa_widths():
    """Tensor-level absmax scaling puts N(0, sigma) gradients in the normal range of either format, so the error
    is the rounding error of a 3-bit against a 2-bit mantissa: relative RMS error below half an ulp
    (2^-(m+1)), and twice as large for E5M2 as for E4M3.  E4M3's smaller range shows only as a few values in
    10^5 flushed to zero; nothing but the absmax element(s) reaches the largest code."""
    rows = {(r["config"], r["linear"], r["fmt"]): r for r in _rows()}
    for (ci, name, fmt), r in rows.items():
        m = 3 if fmt == "e4m3" else 2
        assert 0.25 * 2.0 ** -(m + 1) < r["rel_rms"] < 2.0 ** -(m + 1)
        assert 1 <= r["at_fmax"] <= 200
        if fmt == "e4m3":
            other = rows[(ci, name, "e5m2")]
            assert 1.95 < other["rel_rms"] / r["rel_rms"] < 2.05
            assert 1e-6 < r["flushed"] < 5e-5 and r["subnorm"] < 5e-4
            assert other["flushed"] == 0.0 and other["subnorm"] < 1e-7
            # the two scales differ by FMAX(e5m2) / FMAX(e4m3) = 128 exactly
            assert other["scale"] / r["scale"] == 128.0
