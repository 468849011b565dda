"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU: the C oracle on small, ragged
and degenerate inputs, the C ABI's argument checks and launch sequencing (csrc/api.hip compiled for the
host only, kernel launchers replaced by counting stubs), and the index arithmetic of the GEMM launches (the
walk of the workgroup ids over the tiles and the planner that shares a ragged last round of tiles, replayed by
brute force).  GPU code is not instrumented: device sanitizers are
not available on the test machines."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _run(exe):
    p = subprocess.run([exe], env=ENV, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert p.returncode == 0, p.stdout[-3000:]
    assert "AddressSanitizer" not in p.stdout and "runtime error" not in p.stdout, p.stdout[-3000:]
    return p.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fsanitize=address,undefined",
                           "-fno-sanitize-recover=undefined", "-fopenmp", "-ffp-contract=off", "-o", exe,
                           os.path.join(SAN, "oracle_driver.c"), os.path.join(ROOT, "oracle", "llmq_oracle.c"), "-lm"])
    assert "oracle sanitizer driver ok" in _run(exe)


def test_abi_argument_checks_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "abi_san")
    p = subprocess.run([hipcc, "--cuda-host-only", "-O1", "-g", "-std=c++17",
                        "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                        "-Xarch_host", "-fno-sanitize-recover=undefined", "-o", exe,
                        os.path.join(ROOT, "paper_2512_15306_amd", "csrc", "api.hip"),
                        os.path.join(SAN, "abi_driver.hip")], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert p.returncode == 0, p.stdout[-3000:]
    assert "abi sanitizer driver ok" in _run(exe)


def _hipcc_host(tmp_path, name, sources, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / name)
    p = subprocess.run([hipcc, "--cuda-host-only", "-O1", "-g", "-std=c++17",
                        "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                        "-Xarch_host", "-fno-sanitize-recover=undefined", "-I", os.path.join(ROOT, "include"),
                        *extra, "-o", exe, *sources], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert p.returncode == 0, p.stdout[-3000:]
    return exe


def test_tile_walk_and_sharing_plans_by_brute_force(tmp_path):
    """Every tile exactly once for every grid; every K step of every shared tile exactly once, every partial
    result in a slot of its own inside the scratch the plan asks for, for the planner's own rule and for the
    forced modes the GPU tests use (LLMQ_GEMM_SPLIT=1, a<n>)."""
    exe = _hipcc_host(tmp_path, "planner_san", [os.path.join(SAN, "planner_driver.hip")])
    env = dict(ENV, LLMQ_TUNING="1")
    p = subprocess.run([exe], env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert p.returncode == 0 and "planner driver ok" in p.stdout, p.stdout[-3000:]
    assert "AddressSanitizer" not in p.stdout and "runtime error" not in p.stdout, p.stdout[-3000:]


def test_the_brute_force_notices_a_planted_mistake(tmp_path):
    """The same driver built so that its replay of the pieces launch drops the last K step of every last piece
    (-DLLMQ_PLANT_SHORT_PIECES) must fail: the check has teeth."""
    exe = _hipcc_host(tmp_path, "planner_planted", [os.path.join(SAN, "planner_driver.hip")], extra=("-DLLMQ_PLANT_SHORT_PIECES",))
    p = subprocess.run([exe], env=dict(ENV, LLMQ_TUNING="1"), stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=300)
    assert p.returncode != 0 and "computed 0 times" in p.stdout, p.stdout[-2000:]
