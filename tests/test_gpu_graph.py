"""The library's calls can be captured into a HIP graph (they only launch kernels on the given
stream: no allocation, no memset, no host synchronisation) and every replay reproduces the
eager results bit for bit."""
import numpy as np
import pytest
import torch

import moss_inputs as mi
import paper_2511_05811_amd as moss
from gpu_util import bf16_to_gpu, to_gpu

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


ROW, COL = moss.MOSS_Q_ROW, moss.MOSS_Q_COL


def quant_buffers(rows, cols, dev):
    u8 = torch.uint8
    return dict(q_row=torch.zeros((rows, cols), dtype=u8, device=dev), e_row=torch.zeros((rows, cols // 32), dtype=u8, device=dev),
                q_col=torch.zeros((cols, rows), dtype=u8, device=dev), e_col=torch.zeros((cols, rows // 32), dtype=u8, device=dev),
                s=torch.zeros(1, dtype=torch.float32, device=dev))


@pytest.mark.parametrize("tokens,k,n", [(4096, 4096, 1024),      # X on the one-launch quantizer (1024 tiles), dY on the two-launch path
                                        (1024, 2048, 1536)])     # both on the two-launch path
def test_static_scratch_quantizer_and_gemm_chains_in_a_graph(tokens, k, n):
    """A linear's forward chain (static-scratch quantizer -> block-scaled GEMM) and its weight-gradient chain (both
    groupings of dY and X -> FP32 GEMM), captured once and replayed with new contents in the input buffers: every replay
    gives, bit for bit, what the eager calls with a workspace give on the same contents."""
    dev = torch.device("cuda:0")
    w = to_gpu(mi.config4_weights(n, k, seed=91))
    state = moss.new_wscale_state(dev)
    wq, _ = moss.weight_autoscale_init(w, state)
    s_w = state[4:8].view(torch.float32)                     # s_cur inside the device-resident state

    x = torch.zeros((tokens, k), dtype=torch.bfloat16, device=dev)          # the graph's input buffers
    dy = torch.zeros((tokens, n), dtype=torch.bfloat16, device=dev)
    qx, qdy = quant_buffers(tokens, k, dev), quant_buffers(tokens, n, dev)
    y = torch.zeros((tokens, n), dtype=torch.bfloat16, device=dev)
    dw = torch.zeros((n, k), dtype=torch.float32, device=dev)

    def chain():
        moss.quant_act_2level_noalloc(x, ROW | COL, qx)
        moss.gemm_fp8_mx(qx["q_row"], qx["e_row"], qx["s"], wq, None, s_w, out=y)
        moss.quant_act_2level_noalloc(dy, ROW | COL, qdy)
        moss.gemm_fp8_mx(qdy["q_col"], qdy["e_col"], qdy["s"], qx["q_col"], qx["e_col"], qx["s"], out=dw, out_dtype=torch.float32)

    def load_inputs(seed):
        x.copy_(bf16_to_gpu(mi.heavy_tailed_activation(tokens, k, seed=seed)))
        dy.copy_(bf16_to_gpu(mi.heavy_tailed_activation(tokens, n, seed=seed + 1000)) * 1e-3)

    # everything that asks the runtime a question (the scratch array's address, kernel attributes, occupancy)
    # happens on the first eager call, outside the capture
    load_inputs(1)
    chain()
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chain()
    torch.cuda.synchronize()

    for rep, seed in enumerate((2, 3, 4, 2)):
        print(f"[graph] tokens={tokens} k={k} n={n} replay {rep} seed {seed}", flush=True)
        load_inputs(seed)
        for t in (y, dw, *qx.values(), *qdy.values()):
            t.zero_()                                        # (eager work between the replays)
        graph.replay()
        torch.cuda.synchronize()
        got = dict(y=y.clone(), dw=dw.clone(), **{f"x_{a}": b.clone() for a, b in qx.items()}, **{f"dy_{a}": b.clone() for a, b in qdy.items()})
        # the same contents through the eager entry points with a workspace
        ex = moss.quant_act_2level(x, ROW | COL)
        edy = moss.quant_act_2level(dy, ROW | COL)
        ey = moss.gemm_fp8_mx(ex["q_row"], ex["e_row"], ex["s"], wq, None, s_w)
        edw = moss.gemm_fp8_mx(edy["q_col"], edy["e_col"], edy["s"], ex["q_col"], ex["e_col"], ex["s"], out_dtype=torch.float32)
        torch.cuda.synchronize()
        for a in ("q_row", "e_row", "q_col", "e_col", "s"):
            assert torch.equal(got[f"x_{a}"], ex[a]), (rep, "x", a)
            assert torch.equal(got[f"dy_{a}"], edy[a]), (rep, "dy", a)
        assert torch.equal(got["y"].view(torch.int16), ey.view(torch.int16)), (rep, "y")
        assert torch.equal(got["dw"].view(torch.int32), edw.view(torch.int32)), (rep, "dw")
        assert float(got["x_s"]) > 0 and bool(torch.isfinite(got["dw"]).all())
