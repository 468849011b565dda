"""Build libllmq.so (the gfx950 kernels and their C ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import re
import shutil
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libllmq.so")
# gemm_tiles_*.hip: the tile kernels of one operand-kind pair and layout each (all tile shapes), so that they compile
# side by side; the largest come first.
TILE_SOURCES = ["gemm_tiles_e4m3_e4m3.hip", "gemm_tiles_e5m2_e4m3.hip", "gemm_tiles_e4m3_e5m2.hip", "gemm_tiles_e5m2_e5m2.hip",
                "gemm_tiles_e4m3_e4m3_abt.hip", "gemm_tiles_e4m3_e4m3_bt.hip", "gemm_tiles_e4m3_e4m3_at.hip",
                "gemm_tiles_e5m2_e4m3_abt.hip", "gemm_tiles_e5m2_e4m3_bt.hip", "gemm_tiles_e5m2_e4m3_at.hip",
                "gemm_tiles_bf16_bf16.hip"]
SOURCES = TILE_SOURCES + ["gemm.hip", "gemm_tmajor.hip", "api.hip", "amax.hip", "quantize.hip", "swiglu.hip", "rmsnorm.hip", "calibrate.hip"]
# Sources that hold tile kernels (see check_accumulator_reads).
CHECKED_SOURCES = set(TILE_SOURCES) | {"gemm.hip"}
# packed-fp32 VALU ops are disabled on purpose (they have produced silent wrong results on this
# hardware pool); never add -ffast-math: the scale needs a correctly rounded division.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def check_accumulator_reads(src: str, asm: str) -> None:
    """The tile kernels write their MFMAs out as inline assembly, so the compiler does not know that an
    accumulator read must keep its distance from the MFMA that wrote it.  The kernels' own code keeps it: nothing
    but MFMAs touches the accumulator registers (other than to zero them from an ordinary register) from the first MFMA to the wait states
    behind the K loop (`s_nop 15`).  Code the register allocator adds on its own (copies between the register files, spills of
    accumulators) would not, so any such instruction in that stretch of the generated assembly is a build error."""
    bad = []
    checked = 0
    for m in re.finditer(r"^(_ZN4llmq16gemm_tile_kernel\w*):[^\n]*\n(.*?)^\.Lfunc_end", asm, re.S | re.M):
        name, body = m.group(1), m.group(2)
        code = [l.split(";")[0].strip() for l in body.splitlines()]
        code = [l for l in code if l and not l.endswith(":")]
        mfma = [i for i, l in enumerate(code) if l.startswith("v_mfma_")]
        if not mfma:
            continue                                  # the kernel that only adds up pieces
        checked += 1
        drain = next((i for i in range(mfma[-1], len(code)) if code[i] == "s_nop 15"), None)
        if drain is None:
            bad.append("%s: no wait states behind the last MFMA" % name)
            continue
        for l in code[mfma[0]:drain]:
            # (the zeroing of the accumulators, a write from an ordinary register, may be repeated on the path of a
            # single K step, which follows the K loop in the text)
            if re.fullmatch(r"v_accvgpr_write_b32 a\d+, v\d+", l):
                continue
            if not l.startswith("v_mfma_") and re.search(r"\ba(\d+|\[\d+:\d+\])", l):
                bad.append("%s: %s" % (name, l))
                break
    if not checked:
        raise RuntimeError("%s: no tile kernel found in the generated assembly" % src)
    if bad:
        raise RuntimeError("%s: accumulator registers touched inside the MFMA stretch:\n  %s" % (src, "\n  ".join(bad)))


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    work = tempfile.mkdtemp(prefix="llmq_build_")
    try:
        return _build_in(work, hipcc, verbose)
    finally:
        shutil.rmtree(work, ignore_errors=True)


def _build_in(work: str, hipcc: str, verbose: bool) -> str:
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(work, src.replace(".hip", ".o"))
        cmd = [hipcc] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if src in CHECKED_SOURCES:
            cmd.append("-save-temps=obj")             # keeps the device assembly next to the object
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            print("FAILED: %s\n%s" % (src, out), file=sys.stderr)
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    for src in sorted(CHECKED_SOURCES):
        with open(os.path.join(work, src.replace(".hip", "-hip-amdgcn-amd-amdhsa-gfx950.s"))) as f:
            check_accumulator_reads(src, f.read())
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
