"""The entry point that allocates nothing (llmq_amax_static) against llmq_amax, through the raw C ABI.

Collected last on purpose (the file name sorts after the other test files)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2512_15306_amd import llmq, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _bits(t):
    return int(t.cpu().view(torch.int32).item()) & 0xFFFFFFFF


def test_static_scratch_absmax_matches_the_workspace_call_twice_in_a_row():
    """Two calls in a row on one GPU, the second on a smaller tensor (it leaves most of the first call's
    partial results in the shared array untouched): absmax and scale must be the bits llmq_amax gives with a
    caller workspace, which in turn are the oracle's.  Called through ctypes on the raw symbols."""
    L = llmq.lib()
    stream = torch.cuda.current_stream().cuda_stream
    g = torch.Generator().manual_seed(77)
    big = (torch.randn(40 * 1024 * 1024 + 13, generator=g) * 3.0).to(torch.bfloat16)
    big[31 * 1024 * 1024 + 5] = -977.0                      # the absmax sits in a late block
    small = (torch.randn(70001, generator=g) * 0.01).to(torch.bfloat16)
    ws = torch.full((llmq.llmq_amax_workspace_bytes(),), 0xFF, dtype=torch.uint8, device=DEV)
    for name, host, fmt in (("big", big, llmq.E4M3), ("small", small, llmq.E5M2)):
        print("static absmax:", name, host.numel(), flush=True)
        x = host.to(DEV)
        out = torch.full((4,), -1.0, dtype=torch.float32, device=DEV)       # amax, scale (static); amax, scale (workspace)
        p = out.data_ptr()
        st = L.llmq_amax_static(ctypes.c_void_p(x.data_ptr()), x.numel(), fmt, ctypes.c_void_p(p), ctypes.c_void_p(p + 4),
                                ctypes.c_void_p(stream))
        assert st == 0, llmq.status_string(st)
        st = L.llmq_amax(ctypes.c_void_p(x.data_ptr()), x.numel(), fmt, ctypes.c_void_p(p + 8), ctypes.c_void_p(p + 12),
                         ctypes.c_void_p(ws.data_ptr()), ws.numel(), ctypes.c_void_p(stream))
        assert st == 0, llmq.status_string(st)
        torch.cuda.synchronize()
        got = out.cpu().view(torch.int32).numpy().view(np.uint32)
        assert got[0] == got[2] and got[1] == got[3], (name, got)
        a = oracle.amax_bf16(synth.bf16_bits(host))
        assert got[0] == np.float32(a).view(np.uint32) and got[1] == np.float32(oracle.scale(a, fmt)).view(np.uint32)
    # argument errors come back as status codes before anything is launched
    x = small.to(DEV)
    out = torch.zeros(2, dtype=torch.float32, device=DEV)
    assert L.llmq_amax_static(None, 8, 0, ctypes.c_void_p(out.data_ptr()), None, None) == -1
    assert L.llmq_amax_static(ctypes.c_void_p(x.data_ptr()), 0, 0, ctypes.c_void_p(out.data_ptr()), None, None) == -2
    assert L.llmq_amax_static(ctypes.c_void_p(x.data_ptr()), 1 << 40, 0, ctypes.c_void_p(out.data_ptr()), None, None) == -2
    assert L.llmq_amax_static(ctypes.c_void_p(x.data_ptr()), 8, 7, ctypes.c_void_p(out.data_ptr()), None, None) == -4
    assert L.llmq_amax_static(ctypes.c_void_p(x.data_ptr() + 2), 8, 0, ctypes.c_void_p(out.data_ptr()), None, None) == -3
