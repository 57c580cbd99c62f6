"""The library's calls can be captured into a HIP graph (they only launch kernels on the given
stream: no allocation, no memset, no host synchronisation) and every replay reproduces the
eager results bit for bit."""
import numpy as np
import pytest
import torch

import paper_2511_05811_amd as moss

pytestmark = pytest.mark.gpu


def test_quantize_gemm_update_chain_in_a_graph():
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(77)
    T, K, N = 4096, 2048, 1024
    u8, f32, bf16 = torch.uint8, torch.float32, torch.bfloat16
    x = torch.randn((T, K), generator=gen, device=dev, dtype=f32).to(bf16)
    dy = (torch.randn((T, N), generator=gen, device=dev, dtype=f32) * 1e-3).to(bf16)
    w0 = torch.randn((N, K), generator=gen, device=dev, dtype=f32) * 0.02
    both = moss.MOSS_Q_ROW | moss.MOSS_Q_COL
    lib = moss.load()

    def qbuf(r, c):
        return dict(q_row=torch.empty((r, c), dtype=u8, device=dev), e_row=torch.empty((r, c // 32), dtype=u8, device=dev),
                    q_col=torch.empty((c, r), dtype=u8, device=dev), e_col=torch.empty((c, r // 32), dtype=u8, device=dev),
                    s=torch.empty(1, dtype=f32, device=dev))

    class Run:
        def __init__(self):
            self.w, self.m, self.v = w0.clone(), torch.zeros_like(w0), torch.zeros_like(w0)
            self.state = moss.new_wscale_state(dev)
            self.wq = torch.empty((N, K), dtype=u8, device=dev)
            self.wq_t = torch.empty((K, N), dtype=u8, device=dev)
            self.ws_w = torch.empty(max(16, lib.moss_weight_workspace_bytes(N, K)), dtype=u8, device=dev)
            self.ws_q = torch.empty(max(16, lib.moss_quant_workspace_bytes(T, max(K, N), 3)), dtype=u8, device=dev)
            moss.weight_autoscale_init(self.w, self.state, wq=self.wq, wq_t=self.wq_t, workspace=self.ws_w)
            self.s_w = self.state[4:8].view(f32)
            self.qx, self.qdy = qbuf(T, K), qbuf(T, N)
            self.y = torch.empty((T, N), dtype=bf16, device=dev)
            self.dx = torch.empty((T, K), dtype=bf16, device=dev)
            self.dw = torch.empty((N, K), dtype=f32, device=dev)
            # the optimizer arguments of steps 1..3 live in host memory the calls read at launch time
            b1, b2 = float(np.float32(0.9)), float(np.float32(0.95))
            self.args = [moss.AdamWArgs(3e-4, 0.9, 0.95, 1e-8, 0.1, 1.0 - b1, 1.0 - b2, 1.0 - b1 ** t, 1.0 - b2 ** t, 1.0, 500, t)
                         for t in (1, 2, 3)]

        def step(self, t):
            moss.quant_act_2level(x, both, out=self.qx, workspace=self.ws_q)
            moss.gemm_fp8_mx(self.qx["q_row"], self.qx["e_row"], self.qx["s"], self.wq, None, self.s_w, out=self.y)
            moss.quant_act_2level(dy, both, out=self.qdy, workspace=self.ws_q)
            moss.gemm_fp8_mx(self.qdy["q_row"], self.qdy["e_row"], self.qdy["s"], self.wq_t, None, self.s_w, out=self.dx)
            moss.gemm_fp8_mx(self.qdy["q_col"], self.qdy["e_col"], self.qdy["s"], self.qx["q_col"], self.qx["e_col"],
                             self.qx["s"], out=self.dw, out_dtype=f32)
            moss.weight_autoscale_cast(self.w, self.m, self.v, self.dw, self.args[t - 1], self.state, wq=self.wq,
                                       wq_t=self.wq_t, workspace=self.ws_w)

        def snapshot(self):
            torch.cuda.synchronize()
            return [t.clone() for t in (self.y, self.dx, self.dw, self.w, self.m, self.v, self.wq, self.wq_t, self.state)]

    eager = Run()
    want = []
    for t in (1, 2, 3):
        eager.step(t)
        want.append(eager.snapshot())

    graphed = Run()
    graphs = []
    side = torch.cuda.Stream()
    for t in (1, 2, 3):              # one graph per optimizer step (the step number is a launch-time argument)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            graphed.step(t)
        graphs.append(g)
    # capture launched nothing: rewind to the initial state, then replay with eager work in between
    fresh = Run()
    for dst, src in zip((graphed.w, graphed.m, graphed.v, graphed.wq, graphed.wq_t, graphed.state),
                        (fresh.w, fresh.m, fresh.v, fresh.wq, fresh.wq_t, fresh.state)):
        dst.copy_(src)
    for t in (1, 2, 3):
        graphs[t - 1].replay()
        got = graphed.snapshot()
        scratch = torch.randn(1 << 20, device=dev).sum().item()      # unrelated eager work and a synchronisation
        assert np.isfinite(scratch)
        for a, b, name in zip(got, want[t - 1], ("y", "dx", "dw", "w", "m", "v", "wq", "wq_t", "state")):
            assert torch.equal(a, b), (t, name)


def test_producer_chain_in_a_graph():
    """SwiGLU (which clears and fills its maximum word with kernels, no memset) followed by the quantizer that
    takes the word: captured once, replayed on changing inputs, each replay equal to the eager result."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(78)
    rows, cols = 1024, 1536
    bf16 = torch.bfloat16
    both = moss.MOSS_Q_ROW | moss.MOSS_Q_COL
    g = torch.empty((rows, cols), dtype=bf16, device=dev)
    u = torch.empty((rows, cols), dtype=bf16, device=dev)
    d = torch.empty((rows, cols), dtype=bf16, device=dev)

    def fill(seed_scale):
        g.copy_((torch.randn((rows, cols), generator=gen, device=dev) * seed_scale).to(bf16))
        u.copy_(torch.randn((rows, cols), generator=gen, device=dev).to(bf16))
        d.copy_((torch.randn((rows, cols), generator=gen, device=dev) * 1e-2).to(bf16))

    class Bufs:
        def __init__(self):
            self.h = torch.empty((rows, cols), dtype=bf16, device=dev)
            self.dg, self.du = torch.empty_like(self.h), torch.empty_like(self.h)
            self.w = [torch.empty(1, dtype=torch.int32, device=dev) for _ in range(3)]
            self.q = None

        def run(self):
            moss.swiglu_bf16(g, u, h=self.h, absmax_bits=self.w[0])
            self.q = moss.quant_act_2level_given_max(self.h, self.w[0], both, out=self.q)
            moss.swiglu_bf16_backward(g, u, d, d_gate=self.dg, d_up=self.du, d_gate_absmax_bits=self.w[1], d_up_absmax_bits=self.w[2])

        def snapshot(self):
            torch.cuda.synchronize()
            return [t.clone() for t in (self.h, self.dg, self.du, *self.w, self.q["q_row"], self.q["e_row"], self.q["q_col"],
                                        self.q["e_col"], self.q["s"])]

    fill(1.0)
    graphed = Bufs()
    graphed.run()                        # allocates the quantizer's outputs once, outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=torch.cuda.Stream()):
        graphed.run()
    eager = Bufs()
    for scale in (0.5, 3.0, 8.0):
        fill(scale)
        eager.run()
        want = eager.snapshot()
        graph.replay()
        got = graphed.snapshot()
        assert np.isfinite(torch.randn(1 << 18, device=dev).sum().item())
        for i, (a, b) in enumerate(zip(got, want)):
            assert torch.equal(a, b), (scale, i)
