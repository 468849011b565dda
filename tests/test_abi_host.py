"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol that
include/llmq.h declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2512_15306_amd import llmq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "llmq.h")).read()
    declared = set(re.findall(r"\b(llmq_[a-z0-9_]+)\s*\(", header))
    declared -= {"llmq_status", "llmq_fp8_format"}
    assert declared == set(llmq.EXPORTS)
    L = llmq.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert llmq.version() >= 100
    assert llmq.status_string(0) == "ok"
    for st in range(-7, 0):
        assert llmq.status_string(st) not in ("ok", "unknown status")


def test_workspace_layout():
    M, N, K = 256, 1024, 512
    offs = llmq.llmq_fp8_linear_workspace_offsets(M, N, K)
    sizes = [M * K, M * K, N * K, N * K, M * N, M * N]
    total = llmq.llmq_fp8_linear_workspace_bytes(M, N, K)
    compact = llmq.llmq_fp8_linear_workspace_bytes_no_transpose(M, N, K)
    assert offs[0] == 0 and all(o % 256 == 0 for o in offs)
    spans = sorted((o, o + n) for o, n in zip(offs, sizes))
    for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
        assert a1 <= b0                                         # no two copies overlap
    assert spans[-1][1] <= total
    # row-major copies and the scratch (12 KB) come first: a workspace without transposed copies is a prefix
    assert max(offs[i] + sizes[i] for i in (0, 2, 4)) + 12288 <= compact <= min(offs[i] for i in (1, 3, 5))
    assert compact < total and total - compact >= sum(sizes[1::2])
    # ragged sizes are padded to 256-byte boundaries
    offs = llmq.llmq_fp8_linear_workspace_offsets(3, 5, 7)
    assert all(o % 256 == 0 for o in offs) and len(set(offs)) == 6
    assert llmq.llmq_fp8_linear_workspace_bytes(0, 1, 1) == 0
    assert llmq.llmq_fp8_linear_workspace_bytes_shared(1, 1, 0) == 0
    # the section for the pieces of shared tiles comes behind everything else and is as large as the largest
    # of the three contractions asks for (nothing for shapes that never share)
    assert llmq.llmq_fp8_linear_workspace_bytes_shared(M, N, K) == total
    big = (16384, 5120, 7168)
    want = max(llmq.llmq_fp8_gemm_scratch_bytes(*rct) for rct in ((16384, 5120, 7168), (16384, 7168, 5120), (5120, 7168, 16384)))
    assert want > 0 and llmq.llmq_fp8_linear_workspace_bytes_shared(*big) == llmq.llmq_fp8_linear_workspace_bytes(*big) + want
    assert llmq.llmq_fp8_linear_workspace_bytes_no_transpose(1, 0, 1) == 0


def test_argument_errors_are_reported_before_any_launch():
    L = llmq.lib()
    ok_ptr = 0x10000          # never dereferenced: every call below fails validation on the host
    odd_ptr = 0x10008
    n = ctypes.c_size_t
    aw = llmq.llmq_amax_workspace_bytes()
    assert aw >= 1024
    assert L.llmq_amax(None, 8, 0, ok_ptr, ok_ptr, ok_ptr, n(aw), None) == -1
    assert L.llmq_amax(ok_ptr, 8, 0, None, ok_ptr, ok_ptr, n(aw), None) == -1
    assert L.llmq_amax(ok_ptr, 8, 0, ok_ptr, ok_ptr, None, n(aw), None) == -1
    assert L.llmq_amax(ok_ptr, 0, 0, ok_ptr, ok_ptr, ok_ptr, n(aw), None) == -2
    assert L.llmq_amax(ok_ptr, 8, 2, ok_ptr, ok_ptr, ok_ptr, n(aw), None) == -4
    assert L.llmq_amax_static(None, 8, 0, ok_ptr, ok_ptr, None) == -1
    assert L.llmq_amax_static(ok_ptr, 8, 0, None, ok_ptr, None) == -1
    assert L.llmq_amax_static(ok_ptr, 0, 0, ok_ptr, ok_ptr, None) == -2
    assert L.llmq_amax_static(ok_ptr, n(1 << 40), 0, ok_ptr, ok_ptr, None) == -2
    assert L.llmq_amax_static(ok_ptr, 8, 2, ok_ptr, ok_ptr, None) == -4
    assert L.llmq_amax_static(odd_ptr, 8, 0, ok_ptr, ok_ptr, None) == -3
    assert L.llmq_amax(odd_ptr, 8, 0, ok_ptr, ok_ptr, ok_ptr, n(aw), None) == -3
    assert L.llmq_amax(ok_ptr, 8, 0, ok_ptr + 2, ok_ptr, ok_ptr, n(aw), None) == -3
    assert L.llmq_amax(ok_ptr, 8, 0, ok_ptr, ok_ptr, ok_ptr, n(aw - 1), None) == -5
    assert L.llmq_quantize_fp8(ok_ptr, 4, 4, None, 0, ok_ptr, ok_ptr, None) == -1
    assert L.llmq_quantize_fp8(ok_ptr, 0, 4, ok_ptr, 0, ok_ptr, ok_ptr, None) == -2
    assert L.llmq_quantize_fp8(ok_ptr, 4, -1, ok_ptr, 0, ok_ptr, ok_ptr, None) == -2
    assert L.llmq_quantize_fp8(ok_ptr, 4, 4, ok_ptr, 7, ok_ptr, ok_ptr, None) == -4
    assert L.llmq_quantize_fp8(ok_ptr, 4, 4, ok_ptr, 0, odd_ptr, ok_ptr, None) == -3
    assert L.llmq_fp8_gemm_tn(ok_ptr, 0, None, 0, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, 0, None, None) == -1
    assert L.llmq_fp8_gemm_tn(ok_ptr, 0, ok_ptr, 0, 16, 0, 16, ok_ptr, ok_ptr, ok_ptr, 0, None, None) == -2
    assert L.llmq_fp8_gemm_tn(ok_ptr, 3, ok_ptr, 0, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, 0, None, None) == -4
    assert L.llmq_fp8_gemm_tn(ok_ptr, 0, ok_ptr, 0, 16, 16, 16, ok_ptr, ok_ptr, odd_ptr, 0, None, None) == -3
    L.llmq_fp8_gemm.restype = ctypes.c_int
    assert L.llmq_fp8_gemm(ok_ptr, 0, 1, None, 0, 1, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, 0, None, None) == -1
    assert L.llmq_fp8_gemm(ok_ptr, 0, 1, ok_ptr, 0, 1, 16, 0, 16, ok_ptr, ok_ptr, ok_ptr, 0, None, None) == -2
    assert L.llmq_fp8_gemm(ok_ptr, 0, 1, ok_ptr, 5, 0, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, 0, None, None) == -4
    assert L.llmq_fp8_gemm(odd_ptr, 0, 0, ok_ptr, 0, 1, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, 0, None, None) == -3
    assert L.llmq_fp8_gemm(ok_ptr, 0, 3, ok_ptr, 0, 0, 16, 16, 128, ok_ptr, ok_ptr, ok_ptr, 0, None, None) == -7              # no such layout
    assert L.llmq_fp8_gemm(ok_ptr, 0, 0, ok_ptr, 0, -1, 16, 16, 128, ok_ptr, ok_ptr, ok_ptr, 0, None, None) == -7
    assert L.llmq_fp8_gemm(ok_ptr, 0, 2, ok_ptr, 0, 0, 16, 16, 192, ok_ptr, ok_ptr, ok_ptr, 0, None, None) == -2              # slabs are 128 contraction bytes
    ws = 0x100000
    need = llmq.llmq_fp8_linear_workspace_bytes(16, 16, 16)
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, None, n(need), 0, None) == -1
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, ws, n(need - 1), 0, None) == -5
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, ws + 16, n(need), 0, None) == -3
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, ws, n(need), 512, None) == -7
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, ws, n(need), 256 | 64, None) == -7  # slabs are a layout of the transposed copies
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, ws, n(need), 128 | 64, None) == -7  # shared tiles need the transposed copies
    big = (16384, 5120, 7168)                                   # a shape whose weight gradient shares tiles
    shared, plain = llmq.llmq_fp8_linear_workspace_bytes_shared(*big), llmq.llmq_fp8_linear_workspace_bytes(*big)
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, *big, ok_ptr, ok_ptr, ok_ptr, None, ws, n(plain), 128, None) == -5
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, *big, ok_ptr, ok_ptr, ok_ptr, None, ws, n(shared - 1), 128, None) == -5
    small = llmq.llmq_fp8_linear_workspace_bytes_no_transpose(16, 16, 16)
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, ws, n(small), 0, None) == -5
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, ws, n(small - 1), 64, None) == -5
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, ws, n(need), 8 | 1, None) == -7      # JIT and REUSE of one operand
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, ws, n(need), 32, None) == -7         # dY is no operand of the forward call
    assert L.llmq_fp8_linear_wgrad(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, 1, ok_ptr, 0, ws, n(need), 16, None) == -7
    assert L.llmq_fp8_linear_fwd(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, ws, n(need), 4, None) == -7
    assert L.llmq_fp8_linear_fwd(None, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, ok_ptr, None, ws, n(need), 0, None) == -1
    assert L.llmq_fp8_linear_dgrad(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, 5, ok_ptr, None, ws, n(need), 0, None) == -4
    assert L.llmq_fp8_linear_dgrad(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, 1, ok_ptr, None, ws, n(need), 1, None) == -7
    assert L.llmq_fp8_linear_dgrad(ok_ptr, ok_ptr, 16, 0, 16, ok_ptr, ok_ptr, 1, ok_ptr, None, ws, n(need), 0, None) == -2
    assert L.llmq_fp8_linear_wgrad(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, 1, None, 0, ws, n(need), 0, None) == -1
    assert L.llmq_fp8_linear_wgrad(ok_ptr, ok_ptr, 16, 16, 16, ok_ptr, ok_ptr, 1, ok_ptr, 0, ws, n(need), 2, None) == -7


def test_argument_errors_of_the_producer_and_baseline_entry_points():
    L = llmq.lib()
    ok, odd = 0x10000, 0x10008
    n = ctypes.c_size_t
    f = ctypes.c_float
    sw = llmq.llmq_swiglu_workspace_bytes(64, 256)
    assert sw >= 4 and llmq.llmq_swiglu_workspace_bytes(0, 8) == 0 and llmq.llmq_swiglu_workspace_bytes(8, 1 << 24) == 0
    assert L.llmq_swiglu_fwd(None, 64, 256, ok, 0, ok, ok, ok, n(sw), None) == -1
    assert L.llmq_swiglu_fwd(ok, 64, 256, ok, 0, None, ok, ok, n(sw), None) == -1
    assert L.llmq_swiglu_fwd(ok, 64, 0, ok, 0, ok, ok, ok, n(sw), None) == -2
    assert L.llmq_swiglu_fwd(ok, 64, 256, ok, 2, ok, ok, ok, n(sw), None) == -4
    assert L.llmq_swiglu_fwd(odd, 64, 256, ok, 0, ok, ok, ok, n(sw), None) == -3
    assert L.llmq_swiglu_fwd(ok, 64, 256, ok, 0, ok, ok, odd, n(sw), None) == -3          # scratch: 16-byte aligned
    assert L.llmq_swiglu_fwd(ok, 64, 256, ok, 0, ok, ok, ok, n(sw - 1), None) == -5
    assert L.llmq_swiglu_fwd_fp8(ok, 64, 256, None, 0, ok, ok, None, None) == -1
    assert L.llmq_swiglu_fwd_fp8(ok, 64, 256, ok, 0, None, ok, None, None) == -1
    assert L.llmq_swiglu_fwd_fp8(ok, 64, 256, ok, 5, ok, ok, None, None) == -4
    assert L.llmq_swiglu_fwd_fp8(ok, 64, 256, ok, 0, ok, odd, None, None) == -3
    assert L.llmq_swiglu_fwd_fp8_slabs(ok, 128, 256, ok, 0, ok, None, None, None) == -1           # q_t is required
    assert L.llmq_swiglu_fwd_fp8_slabs(ok, 64, 256, ok, 0, ok, ok, None, None) == -2              # whole 128 x 256 tiles only
    assert L.llmq_swiglu_fwd_fp8_slabs(ok, 128, 264, ok, 0, ok, ok, None, None) == -2
    assert L.llmq_swiglu_fwd_fp8_slabs(ok, 1 << 17, 1 << 14, ok, 0, ok, ok, None, None) == -2     # 2^31 elements: not kept in slabs
    assert L.llmq_swiglu_fwd_fp8_slabs(ok, 128, 256, ok, 5, ok, ok, None, None) == -4
    assert L.llmq_swiglu_fwd_fp8_slabs(ok, 128, 256, ok, 0, ok, odd, None, None) == -3
    assert L.llmq_swiglu_bwd(ok, None, 64, 256, ok, 1, ok, ok, ok, n(sw), None) == -1
    assert L.llmq_swiglu_bwd(ok, ok, -1, 256, ok, 1, ok, ok, ok, n(sw), None) == -2
    assert L.llmq_swiglu_bwd(ok, ok, 64, 256, ok, 1, ok, ok, ok, n(0), None) == -5
    rw = llmq.llmq_rmsnorm_workspace_bytes(64)
    assert rw >= 4 and llmq.llmq_rmsnorm_workspace_bytes(0) == 0
    assert L.llmq_rmsnorm_fwd(None, None, ok, 64, 256, f(1e-6), None, ok, ok, 0, ok, ok, ok, n(rw), None) == -1
    assert L.llmq_rmsnorm_fwd(ok, ok, ok, 64, 256, f(1e-6), None, ok, ok, 0, ok, ok, ok, n(rw), None) == -1   # x without res_out
    assert L.llmq_rmsnorm_fwd(ok, None, ok, 64, 256, f(-1.0), None, ok, ok, 0, ok, ok, ok, n(rw), None) == -2
    assert L.llmq_rmsnorm_fwd(ok, None, ok, 64, 256, f(float("nan")), None, ok, ok, 0, ok, ok, ok, n(rw), None) == -2
    assert L.llmq_rmsnorm_fwd(ok, None, ok, 64, 1 << 24, f(1e-6), None, ok, ok, 0, ok, ok, ok, n(rw), None) == -2
    assert L.llmq_rmsnorm_fwd(ok, None, ok, 64, 256, f(1e-6), None, ok, ok, 3, ok, ok, ok, n(rw), None) == -4
    assert L.llmq_rmsnorm_fwd(ok, None, ok, 64, 256, f(1e-6), None, odd, ok, 0, ok, ok, ok, n(rw), None) == -3
    assert L.llmq_rmsnorm_fwd(ok, None, ok, 64, 256, f(1e-6), None, ok, ok, 0, ok, ok, ok, n(rw - 1), None) == -5
    assert L.llmq_rmsnorm_apply_fp8(ok, ok, None, 64, 256, ok, 0, ok, ok, None, None) == -1
    assert L.llmq_rmsnorm_apply_fp8(ok, ok, odd, 64, 256, ok, 0, ok, ok, None, None) == -3        # rstd: 16-byte aligned
    assert L.llmq_rmsnorm_apply_fp8(ok, ok, ok, 64, 256, ok, 9, ok, ok, None, None) == -4
    assert L.llmq_rmsnorm_apply_fp8_slabs(ok, ok, ok, 128, 256, ok, 0, ok, None, None, None) == -1
    assert L.llmq_rmsnorm_apply_fp8_slabs(ok, ok, ok, 64, 256, ok, 0, ok, ok, None, None) == -2
    assert L.llmq_rmsnorm_apply_fp8_slabs(ok, ok, ok, 128, 384, ok, 0, ok, ok, None, None) == -2
    assert L.llmq_rmsnorm_apply_fp8_slabs(ok, ok, odd, 128, 256, ok, 0, ok, ok, None, None) == -3
    assert L.llmq_rmsnorm_apply_fp8_slabs(ok, ok, ok, 128, 256, ok, 7, ok, ok, None, None) == -4
    assert L.llmq_scale_from_amax(None, 0, ok, None) == -1
    assert L.llmq_scale_from_amax(ok, 4, ok, None) == -4
    assert L.llmq_scale_from_amax(ok, 0, ok + 2, None) == -3
    assert L.llmq_bf16_gemm_tn(ok, None, 16, 16, 16, ok, 0, None) == -1
    assert L.llmq_bf16_gemm_tn(ok, ok, 16, 16, 0, ok, 0, None) == -2
    assert L.llmq_bf16_gemm_tn(ok, odd, 16, 16, 16, ok, 0, None) == -3


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(8, dtype=torch.bfloat16)
    a = torch.zeros(1)
    with pytest.raises(ValueError):
        llmq.llmq_amax(x, 0, a, a, torch.zeros(4096, dtype=torch.uint8))
