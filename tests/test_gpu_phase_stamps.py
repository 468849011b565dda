"""The stamped build of the GEMM tile kernel (llmq_calibrate_gemm_phases) gives the bytes of llmq_fp8_gemm_tn and
stamps that are ordered in time."""
import pytest
import torch

from paper_2512_15306_amd import llmq
from gpu_common import DEV, f32_bits
from test_gpu_gemm import _rand_codes, _scales

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("ieee", [True, False])
def test_stamped_kernel_computes_the_same_tensor(ieee):
    R, C, T = 3 * 256, 2 * 256, 640
    A = torch.from_numpy(_rand_codes((R, T), 0, 61)).to(DEV)
    B = torch.from_numpy(_rand_codes((C, T), 0, 62)).to(DEV)
    dsa, dsb = _scales(1.7, 0.6)
    want = torch.empty((R, C), dtype=torch.bfloat16, device=DEV)
    want_amax = torch.zeros(1, dtype=torch.float32, device=DEV)
    llmq.llmq_fp8_gemm_tn(A, 0, B, 0, dsa, dsb, want, False, want_amax)
    c = torch.full((R, C), float("nan"), dtype=torch.bfloat16, device=DEV)
    am = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
    st = llmq.llmq_calibrate_gemm_phases(A, B, dsa, dsb, c, am, ieee).cpu()
    assert torch.equal(c.view(torch.int16), want.view(torch.int16)) and f32_bits(am) == f32_bits(want_amax)
    used = st[st[:, 0] > 0]
    assert used.shape[0] == 6                                  # one row of stamps per tile
    for a, b in ((0, 1), (1, 2), (2, 4), (4, 5), (5, 3)):      # start, prologue, K loop, stores issued, absmax, stores done
        assert (used[:, b] >= used[:, a]).all() and (used[:, 8 + b] >= used[:, 8 + a]).all()
