"""The library under HIP graph capture and under concurrent callers: every entry point only enqueues kernels on
the stream it is given (no allocation, no memset, no synchronisation, no state of its own but the per-GPU scratch
of llmq_amax_static), so a captured sequence of calls must give, on every replay, the bytes the same calls give
eagerly on the inputs of that moment (replayed several times with eager work of the same kernels, changed inputs
and synchronisations in between), and two host threads on two streams must not disturb each other."""
import pytest
import torch

from paper_2512_15306_amd import llmq
from gpu_common import DEV

pytestmark = pytest.mark.gpu

FLAGS = llmq.SHARE_TILES | llmq.SLAB_COPIES


class Block:
    """One linear layer with a SwiGLU in front and an RMSNorm in front of that, all buffers allocated up front."""

    def __init__(self, M, K, N, seed):
        g = torch.Generator(device="cpu").manual_seed(seed)
        r = lambda *shape, std=1.0: (torch.randn(*shape, generator=g) * std).to(torch.bfloat16).to(DEV)
        self.M, self.K, self.N = M, K, N
        self.res, self.xin, self.w_norm = r(M, K), r(M, K, std=0.3), (1.0 + 0.1 * torch.randn(K, generator=g)).to(torch.bfloat16).to(DEV)
        self.gu, self.W, self.dY = r(M, 2 * K, std=1.5), r(N, K, std=0.02), r(M, N, std=1e-3)
        e = lambda *shape, dt=torch.bfloat16: torch.empty(shape, dtype=dt, device=DEV)
        self.res_out, self.y_norm, self.rstd = e(M, K), e(M, K), e(M, dt=torch.float32)
        self.h, self.Y, self.dX, self.dW = e(M, K), e(M, N), e(M, K), e(N, K)
        self.f = torch.zeros(16, dtype=torch.float32, device=DEV)
        self.ws = e(llmq.llmq_fp8_linear_workspace_bytes_shared(M, N, K), dt=torch.uint8)
        self.ws_sw = e(llmq.llmq_swiglu_workspace_bytes(M, K), dt=torch.uint8)
        self.ws_rn = e(llmq.llmq_rmsnorm_workspace_bytes(M), dt=torch.uint8)
        self.ws_am = e(llmq.llmq_amax_workspace_bytes(), dt=torch.uint8)
        self.q, self.qt = e(M, K, dt=torch.uint8), e(M * K, dt=torch.uint8)

    def outputs(self):
        return [self.res_out, self.y_norm, self.rstd, self.h, self.Y, self.dX, self.dW, self.f, self.q, self.qt, self.ws]

    def run(self, with_static_scratch=True):
        f, M, K, N = self.f, self.M, self.K, self.N
        llmq.llmq_rmsnorm_fwd(self.res, self.xin, self.w_norm, 1e-6, self.res_out, self.y_norm, self.rstd, llmq.E4M3, f[0:1], f[1:2], self.ws_rn)
        llmq.llmq_swiglu_fwd(self.gu, self.h, llmq.E4M3, f[2:3], f[3:4], self.ws_sw)
        # X of the linear is the SwiGLU output with the scale the SwiGLU delivered; W and dY are scaled inside the calls
        llmq.llmq_fp8_linear_fwd(self.h, self.W, M, N, K, f[3:4], f[4:5], self.Y, f[5:6], self.ws, FLAGS | llmq.JIT_W)
        llmq.llmq_fp8_linear_dgrad(self.dY, None, M, N, K, f[6:7], f[4:5], llmq.E5M2, self.dX, f[7:8], self.ws,
                                   FLAGS | llmq.JIT_DY | llmq.REUSE_W)
        llmq.llmq_fp8_linear_wgrad(None, None, M, N, K, f[6:7], f[3:4], llmq.E5M2, self.dW, False, self.ws,
                                   FLAGS | llmq.REUSE_X | llmq.REUSE_DY)
        llmq.llmq_amax(self.dX, llmq.E5M2, f[8:9], f[9:10], self.ws_am)
        if with_static_scratch:              # one scratch array per GPU: calls that overlap on one GPU would race
            llmq.llmq_amax_static(self.Y, llmq.E4M3, f[10:11], f[11:12])
        if M % 128 == 0 and K % 256 == 0:
            llmq.llmq_swiglu_fwd_fp8_slabs(self.gu, f[3:4], llmq.E4M3, self.q, self.qt, None)
        else:
            llmq.llmq_swiglu_fwd_fp8(self.gu, f[3:4], llmq.E4M3, self.q, self.qt, None)

    def poison(self):
        for t in self.outputs():
            if t.dtype == torch.float32:
                t.fill_(-3.0)
            else:
                t.view(torch.uint8).fill_(0xA5)

    def new_inputs(self, k):
        self.gu.mul_(-1.0 if k % 2 else 0.5)
        self.dY.mul_(2.0)
        self.W.add_(0.001 * k)
        self.res.mul_(1.25)


@pytest.mark.parametrize("M,K,N", [(256, 512, 1024), (4096, 3072, 3072), (96, 40, 56)])
def test_captured_calls_replay_the_eager_bytes(M, K, N):
    print("graph replay M=%d K=%d N=%d" % (M, K, N), flush=True)
    b = Block(M, K, N, 5 + M)
    b.run()                                   # first use: kernels loaded, per-device set-up done, outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        b.run()
    other = Block(256, 256, 256, 99)          # eager work of the same kernels between the replays
    for k in range(4):
        b.new_inputs(k)
        b.poison()
        b.run()
        torch.cuda.synchronize()
        want = [t.clone() for t in b.outputs()]
        b.poison()
        other.run()
        torch.cuda.synchronize()
        graph.replay()
        other.run()
        torch.cuda.synchronize()
        for i, (got, ref) in enumerate(zip(b.outputs(), want)):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), "replay %d, output %d differs from the eager call" % (k, i)


def test_two_host_threads_on_two_streams():
    """Two host threads call the library at the same time, each on its own stream with its own buffers and
    workspaces (everything but llmq_amax_static, whose scratch is per GPU): the results are those of the same calls
    made one after the other."""
    import threading
    blocks = [Block(512, 768, 1024, 21), Block(768, 512, 640, 22)]
    want = []
    for b in blocks:
        b.poison()
        b.run(with_static_scratch=False)
        torch.cuda.synchronize()
        want.append([t.clone() for t in b.outputs()])
        b.poison()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    errors = []

    def work(i):
        try:
            with torch.cuda.stream(streams[i]):
                for _ in range(25):
                    blocks[i].run(with_static_scratch=False)
            streams[i].synchronize()
        except Exception as e:           # surfaced below: an exception in a thread would otherwise be lost
            errors.append(repr(e))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=60)
    assert not errors, errors
    assert not any(t.is_alive() for t in threads)
    torch.cuda.synchronize()
    for i, b in enumerate(blocks):
        for j, (got, ref) in enumerate(zip(b.outputs(), want[i])):
            assert torch.equal(got.view(torch.uint8), ref.view(torch.uint8)), "thread %d output %d" % (i, j)
