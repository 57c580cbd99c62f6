"""The library's calls under HIP graph capture: a linear's forward chain (static-scratch quantizer -> block-scaled
GEMM) and its weight-gradient chain (both groupings of dY and X -> FP32 GEMM) are captured once and replayed with new
contents in the input buffers; every replay gives, bit for bit, what the eager calls give on the same contents.
Between the replays the program does eager work of its own and synchronises (a graph that is only right on its first
replay would show here)."""
import pytest
import torch

import moss_inputs as mi
import paper_2511_05811_amd as moss
from gpu_util import bf16_to_gpu, to_gpu

pytestmark = pytest.mark.gpu

ROW, COL = moss.MOSS_Q_ROW, moss.MOSS_Q_COL


def quant_buffers(rows, cols, dev):
    u8 = torch.uint8
    return dict(q_row=torch.zeros((rows, cols), dtype=u8, device=dev), e_row=torch.zeros((rows, cols // 32), dtype=u8, device=dev),
                q_col=torch.zeros((cols, rows), dtype=u8, device=dev), e_col=torch.zeros((cols, rows // 32), dtype=u8, device=dev),
                s=torch.zeros(1, dtype=torch.float32, device=dev))


@pytest.mark.parametrize("tokens,k,n", [(4096, 4096, 1024),      # X on the one-launch quantizer (1024 tiles), dY on the two-launch path
                                        (1024, 2048, 1536)])     # both on the two-launch path
def test_captured_linear_replays_match_eager(tokens, k, n):
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
