"""Python binding of libllmq.so: same names as the C ABI (include/llmq.h), argument marshalling only.

PyTorch supplies device memory and the current HIP stream; every step of the path runs in the
library's kernels.  There is no fallback: a missing library or a missing GPU raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch  # imported first on purpose: the library then binds to the HIP runtime PyTorch loaded

E4M3 = 0
E5M2 = 1
REUSE_X = 1
REUSE_W = 2
REUSE_DY = 4
JIT_X = 8
JIT_W = 16
JIT_DY = 32
NO_TRANSPOSE = 64
SHARE_TILES = 128
SLAB_COPIES = 256
LAYOUT_ROWS, LAYOUT_T_MAJOR, LAYOUT_SLABS = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libllmq.so")
_lib = None

EXPORTS = ["llmq_status_string", "llmq_version", "llmq_amax_workspace_bytes", "llmq_amax", "llmq_amax_static", "llmq_quantize_fp8", "llmq_quantize_fp8_slabs", "llmq_fp8_gemm_tn", "llmq_fp8_gemm", "llmq_fp8_gemm_scratch_bytes", "llmq_fp8_gemm_with_scratch", "llmq_bf16_gemm_tn",
           "llmq_fp8_linear_workspace_bytes", "llmq_fp8_linear_workspace_bytes_no_transpose", "llmq_fp8_linear_workspace_bytes_shared", "llmq_fp8_linear_workspace_offsets",
           "llmq_fp8_linear_fwd", "llmq_fp8_linear_dgrad", "llmq_fp8_linear_wgrad",
           "llmq_scale_from_amax", "llmq_swiglu_workspace_bytes", "llmq_swiglu_fwd", "llmq_swiglu_fwd_fp8", "llmq_swiglu_fwd_fp8_slabs",
           "llmq_swiglu_bwd", "llmq_rmsnorm_workspace_bytes", "llmq_rmsnorm_fwd", "llmq_rmsnorm_apply_fp8", "llmq_rmsnorm_apply_fp8_slabs",
           "llmq_calibrate_mfma", "llmq_calibrate_copy", "llmq_calibrate_gemm_phases_bytes", "llmq_calibrate_gemm_phases"]


class LlmqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %d (%s)" % (where, status, status_string(status)))


def lib() -> ctypes.CDLL:
    """Load libllmq.so (built in-tree by paper_2512_15306_amd/build.py); raise if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libllmq.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                           "(expected at %s)" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i64, sz, i32 = c.c_void_p, c.c_int64, c.c_size_t, c.c_int
    L.llmq_status_string.restype = c.c_char_p
    L.llmq_status_string.argtypes = [i32]
    L.llmq_version.restype = i32
    L.llmq_version.argtypes = []
    L.llmq_amax_workspace_bytes.restype = sz
    L.llmq_amax_workspace_bytes.argtypes = []
    L.llmq_amax.restype = i32
    L.llmq_amax.argtypes = [vp, sz, i32, vp, vp, vp, sz, vp]
    L.llmq_amax_static.restype = i32
    L.llmq_amax_static.argtypes = [vp, sz, i32, vp, vp, vp]
    L.llmq_quantize_fp8.restype = i32
    L.llmq_quantize_fp8.argtypes = [vp, i64, i64, vp, i32, vp, vp, vp]
    L.llmq_quantize_fp8_slabs.restype = i32
    L.llmq_quantize_fp8_slabs.argtypes = [vp, i64, i64, vp, i32, vp, vp, vp]
    L.llmq_fp8_gemm_tn.restype = i32
    L.llmq_fp8_gemm_tn.argtypes = [vp, i32, vp, i32, i64, i64, i64, vp, vp, vp, i32, vp, vp]
    L.llmq_fp8_gemm.restype = i32
    L.llmq_fp8_gemm.argtypes = [vp, i32, i32, vp, i32, i32, i64, i64, i64, vp, vp, vp, i32, vp, vp]
    L.llmq_fp8_gemm_scratch_bytes.restype = sz
    L.llmq_fp8_gemm_scratch_bytes.argtypes = [i64, i64, i64]
    L.llmq_fp8_gemm_with_scratch.restype = i32
    L.llmq_fp8_gemm_with_scratch.argtypes = [vp, i32, i32, vp, i32, i32, i64, i64, i64, vp, vp, vp, i32, vp, vp, sz, vp]
    L.llmq_bf16_gemm_tn.restype = i32
    L.llmq_bf16_gemm_tn.argtypes = [vp, vp, i64, i64, i64, vp, i32, vp]
    L.llmq_fp8_linear_workspace_bytes.restype = sz
    L.llmq_fp8_linear_workspace_bytes.argtypes = [i64, i64, i64]
    L.llmq_fp8_linear_workspace_bytes_no_transpose.restype = sz
    L.llmq_fp8_linear_workspace_bytes_no_transpose.argtypes = [i64, i64, i64]
    L.llmq_fp8_linear_workspace_bytes_shared.restype = sz
    L.llmq_fp8_linear_workspace_bytes_shared.argtypes = [i64, i64, i64]
    L.llmq_fp8_linear_workspace_offsets.restype = i32
    L.llmq_fp8_linear_workspace_offsets.argtypes = [i64, i64, i64, c.POINTER(sz)]
    L.llmq_fp8_linear_fwd.restype = i32
    L.llmq_fp8_linear_fwd.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp, vp, vp, sz, i32, vp]
    L.llmq_fp8_linear_dgrad.restype = i32
    L.llmq_fp8_linear_dgrad.argtypes = [vp, vp, i64, i64, i64, vp, vp, i32, vp, vp, vp, sz, i32, vp]
    L.llmq_fp8_linear_wgrad.restype = i32
    L.llmq_fp8_linear_wgrad.argtypes = [vp, vp, i64, i64, i64, vp, vp, i32, vp, i32, vp, sz, i32, vp]
    L.llmq_scale_from_amax.restype = i32
    L.llmq_scale_from_amax.argtypes = [vp, i32, vp, vp]
    L.llmq_swiglu_workspace_bytes.restype = sz
    L.llmq_swiglu_workspace_bytes.argtypes = [i64, i64]
    L.llmq_swiglu_fwd.restype = i32
    L.llmq_swiglu_fwd.argtypes = [vp, i64, i64, vp, i32, vp, vp, vp, sz, vp]
    L.llmq_swiglu_fwd_fp8.restype = i32
    L.llmq_swiglu_fwd_fp8.argtypes = [vp, i64, i64, vp, i32, vp, vp, vp, vp]
    L.llmq_swiglu_fwd_fp8_slabs.restype = i32
    L.llmq_swiglu_fwd_fp8_slabs.argtypes = [vp, i64, i64, vp, i32, vp, vp, vp, vp]
    L.llmq_swiglu_bwd.restype = i32
    L.llmq_swiglu_bwd.argtypes = [vp, vp, i64, i64, vp, i32, vp, vp, vp, sz, vp]
    L.llmq_rmsnorm_workspace_bytes.restype = sz
    L.llmq_rmsnorm_workspace_bytes.argtypes = [i64]
    L.llmq_rmsnorm_fwd.restype = i32
    L.llmq_rmsnorm_fwd.argtypes = [vp, vp, vp, i64, i64, c.c_float, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    L.llmq_rmsnorm_apply_fp8.restype = i32
    L.llmq_rmsnorm_apply_fp8.argtypes = [vp, vp, vp, i64, i64, vp, i32, vp, vp, vp, vp]
    L.llmq_rmsnorm_apply_fp8_slabs.restype = i32
    L.llmq_rmsnorm_apply_fp8_slabs.argtypes = [vp, vp, vp, i64, i64, vp, i32, vp, vp, vp, vp]
    L.llmq_calibrate_mfma.restype = i32
    L.llmq_calibrate_mfma.argtypes = [i32, i32, i32, i32, vp, c.POINTER(c.c_double), vp]
    L.llmq_calibrate_gemm_phases_bytes.restype = sz
    L.llmq_calibrate_gemm_phases_bytes.argtypes = [i64, i64]
    L.llmq_calibrate_gemm_phases.restype = i32
    L.llmq_calibrate_gemm_phases.argtypes = [vp, vp, i64, i64, i64, vp, vp, vp, vp, vp, sz, i32, vp]
    L.llmq_calibrate_copy.restype = i32
    L.llmq_calibrate_copy.argtypes = [vp, vp, sz, vp]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().llmq_status_string(int(status)).decode()


def version() -> int:
    return int(lib().llmq_version())


def _dev(t: Optional[torch.Tensor], dtype=None, name="tensor") -> Optional[int]:
    """Device pointer of a contiguous CUDA/HIP tensor (None passes through as NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must live on the GPU" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, where: str) -> None:
    if status != 0:
        raise LlmqError(status, where)


def llmq_amax_workspace_bytes() -> int:
    return int(lib().llmq_amax_workspace_bytes())


def llmq_amax(x: torch.Tensor, fmt: int, d_amax: torch.Tensor, d_scale: Optional[torch.Tensor],
              ws: torch.Tensor) -> None:
    _check(lib().llmq_amax(_dev(x, torch.bfloat16, "x"), x.numel(), fmt, _dev(d_amax, torch.float32, "d_amax"),
                           _dev(d_scale, torch.float32, "d_scale"), _dev(ws, torch.uint8, "ws"), ws.numel(),
                           _stream()), "llmq_amax")


def llmq_amax_static(x: torch.Tensor, fmt: int, d_amax: torch.Tensor, d_scale: Optional[torch.Tensor]) -> None:
    _check(lib().llmq_amax_static(_dev(x, torch.bfloat16, "x"), x.numel(), fmt, _dev(d_amax, torch.float32, "d_amax"),
                                  _dev(d_scale, torch.float32, "d_scale"), _stream()), "llmq_amax_static")


def llmq_quantize_fp8(x: torch.Tensor, d_scale: torch.Tensor, fmt: int, q: torch.Tensor,
                      q_t: Optional[torch.Tensor]) -> None:
    rows, cols = x.shape
    if q.numel() != rows * cols or (q_t is not None and q_t.numel() != rows * cols):
        raise ValueError("output size does not match the input")
    _check(lib().llmq_quantize_fp8(_dev(x, torch.bfloat16, "x"), rows, cols, _dev(d_scale, torch.float32, "d_scale"),
                                   fmt, _dev(q, torch.uint8, "q"), _dev(q_t, torch.uint8, "q_t"), _stream()),
           "llmq_quantize_fp8")


def llmq_quantize_fp8_slabs(x: torch.Tensor, d_scale: torch.Tensor, fmt: int, q: torch.Tensor, q_t: torch.Tensor) -> None:
    """q_t: rows * cols bytes, the transposed copy as [rows / 128, cols, 128]."""
    rows, cols = x.shape
    if q.numel() != rows * cols or q_t.numel() != rows * cols:
        raise ValueError("output size does not match the input")
    _check(lib().llmq_quantize_fp8_slabs(_dev(x, torch.bfloat16, "x"), rows, cols, _dev(d_scale, torch.float32, "d_scale"),
                                         fmt, _dev(q, torch.uint8, "q"), _dev(q_t, torch.uint8, "q_t"), _stream()),
           "llmq_quantize_fp8_slabs")


def llmq_fp8_gemm_tn(A: torch.Tensor, fmtA: int, B: torch.Tensor, fmtB: int, d_scaleA: torch.Tensor,
                     d_scaleB: torch.Tensor, c: torch.Tensor, accumulate: bool = False,
                     d_amax_c: Optional[torch.Tensor] = None) -> None:
    R, T = A.shape
    C, T2 = B.shape
    if T != T2 or tuple(c.shape) != (R, C):
        raise ValueError("shape mismatch: A %s, B %s, c %s" % (tuple(A.shape), tuple(B.shape), tuple(c.shape)))
    _check(lib().llmq_fp8_gemm_tn(_dev(A, torch.uint8, "A"), fmtA, _dev(B, torch.uint8, "B"), fmtB, R, C, T,
                                  _dev(d_scaleA, torch.float32), _dev(d_scaleB, torch.float32),
                                  _dev(c, torch.bfloat16, "c"), int(bool(accumulate)),
                                  _dev(d_amax_c, torch.float32), _stream()), "llmq_fp8_gemm_tn")


def _operand_dims(t: torch.Tensor, layout: int):
    """(T, rows) of a contraction operand given as [rows, T], [T, rows] or [T / 128, rows, 128]."""
    if layout == LAYOUT_SLABS:
        if t.dim() != 3 or t.shape[2] != 128:
            raise ValueError("an operand in slabs is [T / 128, rows, 128], got %s" % (tuple(t.shape),))
        return t.shape[0] * 128, t.shape[1]
    if t.dim() != 2:
        raise ValueError("operand must be 2-D, got %s" % (tuple(t.shape),))
    return tuple(t.shape) if layout == LAYOUT_T_MAJOR else tuple(t.shape[::-1])


def llmq_fp8_gemm(A: torch.Tensor, fmtA: int, a_t_major: bool, B: torch.Tensor, fmtB: int, b_t_major: bool,
                  d_scaleA: torch.Tensor, d_scaleB: torch.Tensor, c: torch.Tensor, accumulate: bool = False,
                  d_amax_c: Optional[torch.Tensor] = None) -> None:
    """A is [R, T], [T, R] when a_t_major is True / LAYOUT_T_MAJOR, [T / 128, R, 128] when it is LAYOUT_SLABS;
    B likewise."""
    la, lb = int(a_t_major), int(b_t_major)
    T, R = _operand_dims(A, la)
    T2, C = _operand_dims(B, lb)
    if T != T2 or tuple(c.shape) != (R, C):
        raise ValueError("shape mismatch: A %s, B %s, c %s" % (tuple(A.shape), tuple(B.shape), tuple(c.shape)))
    _check(lib().llmq_fp8_gemm(_dev(A, torch.uint8, "A"), fmtA, la, _dev(B, torch.uint8, "B"), fmtB,
                               lb, R, C, T, _dev(d_scaleA, torch.float32),
                               _dev(d_scaleB, torch.float32), _dev(c, torch.bfloat16, "c"), int(bool(accumulate)),
                               _dev(d_amax_c, torch.float32), _stream()), "llmq_fp8_gemm")


def llmq_fp8_gemm_scratch_bytes(R: int, C: int, T: int) -> int:
    return int(lib().llmq_fp8_gemm_scratch_bytes(R, C, T))


def llmq_fp8_gemm_with_scratch(A: torch.Tensor, fmtA: int, a_t_major: bool, B: torch.Tensor, fmtB: int, b_t_major: bool,
                               d_scaleA: torch.Tensor, d_scaleB: torch.Tensor, c: torch.Tensor, accumulate: bool,
                               d_amax_c: Optional[torch.Tensor], scratch: Optional[torch.Tensor]) -> None:
    """llmq_fp8_gemm with scratch (a uint8 tensor or None) for sharing out a ragged last round of tiles."""
    la, lb = int(a_t_major), int(b_t_major)
    T, R = _operand_dims(A, la)
    T2, C = _operand_dims(B, lb)
    if T != T2 or tuple(c.shape) != (R, C):
        raise ValueError("shape mismatch: A %s, B %s, c %s" % (tuple(A.shape), tuple(B.shape), tuple(c.shape)))
    _check(lib().llmq_fp8_gemm_with_scratch(_dev(A, torch.uint8, "A"), fmtA, la, _dev(B, torch.uint8, "B"),
                                            fmtB, lb, R, C, T, _dev(d_scaleA, torch.float32),
                                            _dev(d_scaleB, torch.float32), _dev(c, torch.bfloat16, "c"),
                                            int(bool(accumulate)), _dev(d_amax_c, torch.float32),
                                            _dev(scratch, torch.uint8, "scratch"),
                                            0 if scratch is None else scratch.numel(), _stream()),
           "llmq_fp8_gemm_with_scratch")


def llmq_bf16_gemm_tn(A: torch.Tensor, B: torch.Tensor, c: torch.Tensor, accumulate: bool = False) -> None:
    R, T = A.shape
    C, T2 = B.shape
    if T != T2 or tuple(c.shape) != (R, C):
        raise ValueError("shape mismatch: A %s, B %s, c %s" % (tuple(A.shape), tuple(B.shape), tuple(c.shape)))
    _check(lib().llmq_bf16_gemm_tn(_dev(A, torch.bfloat16, "A"), _dev(B, torch.bfloat16, "B"), R, C, T,
                                   _dev(c, torch.bfloat16, "c"), int(bool(accumulate)), _stream()), "llmq_bf16_gemm_tn")


def llmq_fp8_linear_workspace_bytes(M: int, N: int, K: int) -> int:
    return int(lib().llmq_fp8_linear_workspace_bytes(M, N, K))


def llmq_fp8_linear_workspace_bytes_no_transpose(M: int, N: int, K: int) -> int:
    return int(lib().llmq_fp8_linear_workspace_bytes_no_transpose(M, N, K))


def llmq_fp8_linear_workspace_bytes_shared(M: int, N: int, K: int) -> int:
    return int(lib().llmq_fp8_linear_workspace_bytes_shared(M, N, K))


def llmq_fp8_linear_workspace_offsets(M: int, N: int, K: int) -> Tuple[int, ...]:
    arr = (ctypes.c_size_t * 6)()
    _check(lib().llmq_fp8_linear_workspace_offsets(M, N, K, arr), "llmq_fp8_linear_workspace_offsets")
    return tuple(int(v) for v in arr)


def llmq_fp8_linear_fwd(X, W, M: int, N: int, K: int, d_scale_x, d_scale_w, Y, d_amax_y, ws: torch.Tensor,
                        flags: int = 0) -> None:
    _check(lib().llmq_fp8_linear_fwd(_dev(X, torch.bfloat16, "X"), _dev(W, torch.bfloat16, "W"), M, N, K,
                                     _dev(d_scale_x, torch.float32), _dev(d_scale_w, torch.float32),
                                     _dev(Y, torch.bfloat16, "Y"), _dev(d_amax_y, torch.float32),
                                     _dev(ws, torch.uint8, "ws"), ws.numel(), flags, _stream()),
           "llmq_fp8_linear_fwd")


def llmq_fp8_linear_dgrad(dY, W, M: int, N: int, K: int, d_scale_dy, d_scale_w, fmt_dy: int, dX, d_amax_dx,
                          ws: torch.Tensor, flags: int = 0) -> None:
    _check(lib().llmq_fp8_linear_dgrad(_dev(dY, torch.bfloat16, "dY"), _dev(W, torch.bfloat16, "W"), M, N, K,
                                       _dev(d_scale_dy, torch.float32), _dev(d_scale_w, torch.float32), fmt_dy,
                                       _dev(dX, torch.bfloat16, "dX"), _dev(d_amax_dx, torch.float32),
                                       _dev(ws, torch.uint8, "ws"), ws.numel(), flags, _stream()),
           "llmq_fp8_linear_dgrad")


def llmq_fp8_linear_wgrad(dY, X, M: int, N: int, K: int, d_scale_dy, d_scale_x, fmt_dy: int, dW,
                          accumulate: bool, ws: torch.Tensor, flags: int = 0) -> None:
    _check(lib().llmq_fp8_linear_wgrad(_dev(dY, torch.bfloat16, "dY"), _dev(X, torch.bfloat16, "X"), M, N, K,
                                       _dev(d_scale_dy, torch.float32), _dev(d_scale_x, torch.float32), fmt_dy,
                                       _dev(dW, torch.bfloat16, "dW"), int(bool(accumulate)),
                                       _dev(ws, torch.uint8, "ws"), ws.numel(), flags, _stream()),
           "llmq_fp8_linear_wgrad")


def llmq_scale_from_amax(d_amax: torch.Tensor, fmt: int, d_scale: torch.Tensor) -> None:
    _check(lib().llmq_scale_from_amax(_dev(d_amax, torch.float32, "d_amax"), fmt, _dev(d_scale, torch.float32, "d_scale"),
                                      _stream()), "llmq_scale_from_amax")


def llmq_swiglu_workspace_bytes(M: int, I: int) -> int:
    return int(lib().llmq_swiglu_workspace_bytes(M, I))


def _swiglu_dims(gu: torch.Tensor) -> Tuple[int, int]:
    if gu.dim() != 2 or gu.shape[1] % 2:
        raise ValueError("GU must be [M, 2I]")
    return int(gu.shape[0]), int(gu.shape[1]) // 2


def llmq_swiglu_fwd(gu: torch.Tensor, h: torch.Tensor, fmt: int, d_amax_h: torch.Tensor,
                    d_scale_h: Optional[torch.Tensor], ws: torch.Tensor) -> None:
    M, I = _swiglu_dims(gu)
    if h.numel() != M * I:
        raise ValueError("h must be [M, I]")
    _check(lib().llmq_swiglu_fwd(_dev(gu, torch.bfloat16, "gu"), M, I, _dev(h, torch.bfloat16, "h"), fmt,
                                 _dev(d_amax_h, torch.float32, "d_amax_h"), _dev(d_scale_h, torch.float32, "d_scale_h"),
                                 _dev(ws, torch.uint8, "ws"), ws.numel(), _stream()), "llmq_swiglu_fwd")


def llmq_swiglu_fwd_fp8(gu: torch.Tensor, d_scale_h: torch.Tensor, fmt: int, q: torch.Tensor,
                        q_t: Optional[torch.Tensor], h: Optional[torch.Tensor] = None) -> None:
    M, I = _swiglu_dims(gu)
    if q.numel() != M * I or (q_t is not None and q_t.numel() != M * I) or (h is not None and h.numel() != M * I):
        raise ValueError("output size does not match [M, I]")
    _check(lib().llmq_swiglu_fwd_fp8(_dev(gu, torch.bfloat16, "gu"), M, I, _dev(d_scale_h, torch.float32, "d_scale_h"),
                                     fmt, _dev(q, torch.uint8, "q"), _dev(q_t, torch.uint8, "q_t"),
                                     _dev(h, torch.bfloat16, "h"), _stream()), "llmq_swiglu_fwd_fp8")


def llmq_swiglu_fwd_fp8_slabs(gu: torch.Tensor, d_scale_h: torch.Tensor, fmt: int, q: torch.Tensor,
                              q_t: torch.Tensor, h: Optional[torch.Tensor] = None) -> None:
    M, I = _swiglu_dims(gu)
    if q.numel() != M * I or q_t.numel() != M * I or (h is not None and h.numel() != M * I):
        raise ValueError("output size does not match [M, I]")
    _check(lib().llmq_swiglu_fwd_fp8_slabs(_dev(gu, torch.bfloat16, "gu"), M, I, _dev(d_scale_h, torch.float32, "d_scale_h"),
                                           fmt, _dev(q, torch.uint8, "q"), _dev(q_t, torch.uint8, "q_t"),
                                           _dev(h, torch.bfloat16, "h"), _stream()), "llmq_swiglu_fwd_fp8_slabs")


def llmq_swiglu_bwd(dh: torch.Tensor, gu: torch.Tensor, dgu: torch.Tensor, fmt: int, d_amax_dgu: torch.Tensor,
                    d_scale_dgu: Optional[torch.Tensor], ws: torch.Tensor) -> None:
    M, I = _swiglu_dims(gu)
    if dh.numel() != M * I or dgu.numel() != 2 * M * I:
        raise ValueError("dh must be [M, I] and dGU [M, 2I]")
    _check(lib().llmq_swiglu_bwd(_dev(dh, torch.bfloat16, "dh"), _dev(gu, torch.bfloat16, "gu"), M, I,
                                 _dev(dgu, torch.bfloat16, "dgu"), fmt, _dev(d_amax_dgu, torch.float32, "d_amax_dgu"),
                                 _dev(d_scale_dgu, torch.float32, "d_scale_dgu"), _dev(ws, torch.uint8, "ws"),
                                 ws.numel(), _stream()), "llmq_swiglu_bwd")


def llmq_rmsnorm_workspace_bytes(M: int) -> int:
    return int(lib().llmq_rmsnorm_workspace_bytes(M))


def llmq_rmsnorm_fwd(res: torch.Tensor, x: Optional[torch.Tensor], w: torch.Tensor, eps: float,
                     res_out: Optional[torch.Tensor], y: torch.Tensor, rstd: torch.Tensor, fmt: int,
                     d_amax_y: torch.Tensor, d_scale_y: Optional[torch.Tensor], ws: torch.Tensor) -> None:
    M, C = res.shape
    if w.numel() != C or y.numel() != M * C or rstd.numel() != M or (x is not None and x.numel() != M * C) or \
            (res_out is not None and res_out.numel() != M * C):
        raise ValueError("shape mismatch")
    _check(lib().llmq_rmsnorm_fwd(_dev(res, torch.bfloat16, "res"), _dev(x, torch.bfloat16, "x"),
                                  _dev(w, torch.bfloat16, "w"), M, C, float(eps), _dev(res_out, torch.bfloat16, "res_out"),
                                  _dev(y, torch.bfloat16, "y"), _dev(rstd, torch.float32, "rstd"), fmt,
                                  _dev(d_amax_y, torch.float32, "d_amax_y"), _dev(d_scale_y, torch.float32, "d_scale_y"),
                                  _dev(ws, torch.uint8, "ws"), ws.numel(), _stream()), "llmq_rmsnorm_fwd")


def llmq_rmsnorm_apply_fp8(res: torch.Tensor, w: torch.Tensor, rstd: torch.Tensor, d_scale_y: torch.Tensor, fmt: int,
                           q: torch.Tensor, q_t: Optional[torch.Tensor], y: Optional[torch.Tensor] = None) -> None:
    M, C = res.shape
    if w.numel() != C or rstd.numel() != M or q.numel() != M * C or (q_t is not None and q_t.numel() != M * C) or \
            (y is not None and y.numel() != M * C):
        raise ValueError("shape mismatch")
    _check(lib().llmq_rmsnorm_apply_fp8(_dev(res, torch.bfloat16, "res"), _dev(w, torch.bfloat16, "w"),
                                        _dev(rstd, torch.float32, "rstd"), M, C, _dev(d_scale_y, torch.float32, "d_scale_y"),
                                        fmt, _dev(q, torch.uint8, "q"), _dev(q_t, torch.uint8, "q_t"),
                                        _dev(y, torch.bfloat16, "y"), _stream()), "llmq_rmsnorm_apply_fp8")


def llmq_rmsnorm_apply_fp8_slabs(res: torch.Tensor, w: torch.Tensor, rstd: torch.Tensor, d_scale_y: torch.Tensor,
                                 fmt: int, q: torch.Tensor, q_t: torch.Tensor, y: Optional[torch.Tensor] = None) -> None:
    M, C = res.shape
    if w.numel() != C or rstd.numel() != M or q.numel() != M * C or q_t.numel() != M * C or \
            (y is not None and y.numel() != M * C):
        raise ValueError("shape mismatch")
    _check(lib().llmq_rmsnorm_apply_fp8_slabs(_dev(res, torch.bfloat16, "res"), _dev(w, torch.bfloat16, "w"),
                                              _dev(rstd, torch.float32, "rstd"), M, C,
                                              _dev(d_scale_y, torch.float32, "d_scale_y"), fmt, _dev(q, torch.uint8, "q"),
                                              _dev(q_t, torch.uint8, "q_t"), _dev(y, torch.bfloat16, "y"), _stream()),
           "llmq_rmsnorm_apply_fp8_slabs")


def llmq_calibrate_mfma(fmtA: int, fmtB: int, random_bits: bool, iters: int, d_sink: torch.Tensor) -> float:
    """Enqueue the register-only MFMA loop; returns the FLOP count of the launch."""
    flops = ctypes.c_double(0.0)
    _check(lib().llmq_calibrate_mfma(fmtA, fmtB, int(bool(random_bits)), iters, _dev(d_sink, torch.float32, "d_sink"),
                                     ctypes.byref(flops), _stream()), "llmq_calibrate_mfma")
    return flops.value


def llmq_calibrate_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    if src.numel() * src.element_size() != dst.numel() * dst.element_size():
        raise ValueError("sizes differ")
    _check(lib().llmq_calibrate_copy(_dev(src, None, "src"), _dev(dst, None, "dst"), src.numel() * src.element_size(),
                                     _stream()), "llmq_calibrate_copy")


def llmq_calibrate_gemm_phases(A: torch.Tensor, B: torch.Tensor, d_scaleA: torch.Tensor, d_scaleB: torch.Tensor,
                               c: torch.Tensor, d_amax_c: torch.Tensor, ieee_maximum: bool = True) -> torch.Tensor:
    """Runs the stamped 256 x 256 tile kernel; returns the stamps as an int64 tensor [workgroup ids, 16]
    (rows of ids beyond the number of tiles stay zero)."""
    R, T = A.shape
    C = B.shape[0]
    nbytes = int(lib().llmq_calibrate_gemm_phases_bytes(R, C))
    stamps = torch.zeros((max(nbytes, 8) // 128, 16), dtype=torch.int64, device=A.device)
    _check(lib().llmq_calibrate_gemm_phases(_dev(A, torch.uint8, "A"), _dev(B, torch.uint8, "B"), R, C, T,
                                            _dev(d_scaleA, torch.float32), _dev(d_scaleB, torch.float32),
                                            _dev(c, torch.bfloat16, "c"), _dev(d_amax_c, torch.float32),
                                            _dev(stamps, torch.int64, "stamps"), stamps.numel() * 8,
                                            int(bool(ieee_maximum)), _stream()), "llmq_calibrate_gemm_phases")
    return stamps
