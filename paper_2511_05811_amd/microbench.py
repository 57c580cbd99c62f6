#!/usr/bin/env python3
"""Side tables of the paper re-measured on one MI355X with the library's own kernels.

    python -m paper_2511_05811_amd.microbench scaling   # Table "Time usage to calculate per-tensor scaling factors" (Sec. 3.2)
                                                         # and the interval sweep of the scaling ablation (App.)
    python -m paper_2511_05811_amd.microbench gemm      # Table "Runtime of quantized FP8 GEMM" (Sec. 4.5.1): its seven shapes
    python -m paper_2511_05811_amd.microbench block     # Sec. 4 setting, one decoder block: tokens/s with the linears on the
                                                         # FP8 path vs BF16 GEMMs (attention, norms, SwiGLU: BF16 torch ops)
    python -m paper_2511_05811_amd.microbench producer  # SwiGLU that also hands the tensor maximum to the quantizer (Sec. 3.1,
                                                         # Eq. 2 without the search): one pass over h instead of two
    python -m paper_2511_05811_amd.microbench quant     # the activation quantizer alone, per shape and grouping, beside a plain copy
    python -m paper_2511_05811_amd.microbench limits    # what the machine allows: GEMM rate and shader clock by operand
                                                         # content (power limit), plain device-copy bandwidth

Each mode prints one JSON line.  Inputs are seeded and synthetic; the paper's own figures are
quoted with the hardware they were measured on, as context only.  Everything that is timed
runs in the HIP library; torch supplies memory, streams and events.  (The fidelity figures of
Sec. 3.1 / 4.5.2, SNR of the library's codes against per-tensor and per-group-128 quantization,
are computed by tests/test_gpu_fidelity.py through the CPU oracle, which this package never loads.)
"""
import argparse
import json
import os
import sys


def _events(torch):
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def _time_ms(torch, fn, reps, warmup=2):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        e0, e1 = _events(torch)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1))
    ts.sort()
    return ts[len(ts) // 2], ts[0]


def _adamw_args(moss, t, interval):
    import numpy as np
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.95))
    return moss.AdamWArgs(3e-4, 0.9, 0.95, 1e-8, 0.1, 1.0 - b1, 1.0 - b2, 1.0 - b1 ** t, 1.0 - b2 ** t, 1.0, interval, t)


# Sec. 3.2, table of scaling-factor time: tensor sizes and the paper's H800 figures (ms)
SCALING_SIZES = [((11008, 16384), 0.54, 0.02), ((11008, 8192), 0.32, 0.02), ((4096, 12288), 0.17, 0.02), ((4096, 4096), 0.08, 0.02)]


def scaling(moss, torch, small=False):
    """Per step, just-in-time scaling costs a max-reduction before the cast; here that is the
    step with `interval = 1` (AdamW pass that yields amax, then a second pass that casts with
    the fresh scale).  Automatic scaling predicts the scale from the learning rates, so the
    cast is fused into the one AdamW pass and the scale itself costs a few scalar operations
    inside the kernel that finalises the step."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(40)
    rows_out = []
    sizes = [((1024, 2048), None, None)] if small else SCALING_SIZES
    for (r, c), paper_jit, paper_auto in sizes:
        w = torch.randn((r, c), generator=gen, device=dev, dtype=torch.float32) * 0.02
        m = torch.zeros_like(w); v = torch.zeros_like(w)
        g = torch.randn((r, c), generator=gen, device=dev, dtype=torch.float32) * 1e-3
        wq = torch.empty((r, c), dtype=torch.uint8, device=dev)
        state = moss.new_wscale_state(dev)
        ws = torch.empty(max(16, moss.load().moss_weight_workspace_bytes(r, c)), dtype=torch.uint8, device=dev)
        moss.weight_autoscale_init(w, state, wq=wq, workspace=ws)
        step = [0]

        def one(interval):
            step[0] += 1
            moss.weight_autoscale_cast(w, m, v, g, _adamw_args(moss, step[0], interval), state, wq=wq, workspace=ws)

        auto_ms, _ = _time_ms(torch, lambda: one(0), 8 if small else 12)
        jit_ms, _ = _time_ms(torch, lambda: one(1), 8 if small else 12)
        # the max-reduction alone, as a separate pass over the FP32 weights (what a non-fused
        # just-in-time cast adds): initialisation = max-reduction + cast, minus the cast pass
        init_ms, _ = _time_ms(torch, lambda: moss.weight_autoscale_init(w, state, wq=wq, workspace=ws), 8)
        rows_out.append({"rows": r, "cols": c, "fused_step_auto_ms": round(auto_ms, 4), "step_with_max_reduction_ms": round(jit_ms, 4),
                         "jit_extra_ms_per_step": round(jit_ms - auto_ms, 4), "amax_plus_cast_ms": round(init_ms, 4),
                         "paper_h800_jit_ms": paper_jit, "paper_h800_auto_ms": paper_auto})
        del w, m, v, g, wq
    # interval sweep: amortised cost of the periodic max-reduction and how close the predicted
    # scale stays to the exact one (ratio >= 1 means no overflow is possible)
    sweep = []
    r, c = (512, 1024) if small else (4096, 11008)
    steps = 40 if small else 400
    for interval in ([10, 20] if small else [100, 500, 2000]):
        gen.manual_seed(41)
        w = torch.randn((r, c), generator=gen, device=dev, dtype=torch.float32) * 0.02
        m = torch.zeros_like(w); v = torch.zeros_like(w)
        wq = torch.empty((r, c), dtype=torch.uint8, device=dev)
        state = moss.new_wscale_state(dev)
        ws = torch.empty(max(16, moss.load().moss_weight_workspace_bytes(r, c)), dtype=torch.uint8, device=dev)
        moss.weight_autoscale_init(w, state, wq=wq, workspace=ws)
        worst = 1e30
        for t in range(1, steps + 1):
            g = torch.randn((r, c), generator=gen, device=dev, dtype=torch.float32) * 1e-3
            moss.weight_autoscale_cast(w, m, v, g, _adamw_args(moss, t, interval), state, wq=wq, workspace=ws)
            if t % (steps // 8) == 0:
                st = moss.read_wscale_state(state)
                worst = min(worst, st.s_cur / (st.amax_seen / 448.0))
        st = moss.read_wscale_state(state)
        g = torch.randn((r, c), generator=gen, device=dev, dtype=torch.float32) * 1e-3
        tt = [steps]

        def one_more(iv):
            tt[0] += 1
            moss.weight_autoscale_cast(w, m, v, g, _adamw_args(moss, tt[0], iv), state, wq=wq, workspace=ws)

        extra = _time_ms(torch, lambda: one_more(1), 6)[0] - _time_ms(torch, lambda: one_more(0), 6)[0]
        sweep.append({"interval": interval, "steps": steps, "clipped_count": int(st.clipped_count), "out_of_range_count": int(st.overflow_count),
                      "min_predicted_over_exact_scale": round(worst, 4),
                      "amortised_max_reduction_ms_per_step": round(extra / interval, 5)})
        del w, m, v, wq
    return {"table": "scaling", "unit": "ms", "sizes": rows_out, "interval_sweep": sweep,
            "note": "paper figures: NVIDIA H800, context only"}


# Sec. 4.5.1, table of quantized FP8 GEMM runtime: (M, N, K) and the paper's MOSS time on H800 (ms)
GEMM_SHAPES = [((2048, 7168, 4096), 0.25), ((2048, 7168, 11008), 0.67), ((4096, 2048, 7168), 0.45), ((4096, 4096, 8192), 0.60),
               ((4096, 4096, 12288), 0.72), ((5120, 5120, 10240), 1.04), ((8192, 8192, 8192), 1.98)]


def gemm(moss, torch, small=False):
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(42)
    out_rows = []
    shapes = [((512, 768, 512), None)] if small else GEMM_SHAPES
    for (M, N, K), paper_ms in shapes:
        x = torch.randn((M, K), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        w = (torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02).to(torch.bfloat16)
        qx = moss.quant_act_2level(x, moss.MOSS_Q_ROW)
        state = moss.new_wscale_state(dev)
        wq, _ = moss.weight_autoscale_init(w, state)
        s_w = state[4:8].view(torch.float32)
        y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
        ms, best = _time_ms(torch, lambda: moss.gemm_fp8_mx(qx["q_row"], qx["e_row"], qx["s"], wq, None, s_w, out=y), 10)
        bf_ms, _ = _time_ms(torch, lambda: moss.gemm_bf16_baseline(x, w, out=y), 5)
        q_ms, _ = _time_ms(torch, lambda: moss.quant_act_2level(x, moss.MOSS_Q_ROW, out=qx), 5)
        out_rows.append({"M": M, "N": N, "K": K, "fp8_mx_ms": round(ms, 4), "fp8_mx_tflops": round(2.0 * M * N * K / ms / 1e9, 1),
                         "bf16_hand_gemm_ms": round(bf_ms, 4), "quant_x_ms": round(q_ms, 4), "paper_h800_moss_ms": paper_ms})
    return {"table": "gemm_shapes", "rows": out_rows, "note": "GEMM alone, operands already quantized; paper figures: NVIDIA H800, context only"}


def block(moss, torch, small=False):
    """One training step (forward, backward, optimizer) of one LLaMA-7B-shaped decoder block at batch 2 x
    sequence 4096.  Both arms share the BF16 scaffolding (RMSNorm, rotary embedding, causal scaled-dot-product
    attention, SwiGLU, residuals); only the five linears and their optimizer differ."""
    import time
    from . import block as blk
    sz = blk.sizes_small() if small else blk.sizes_7b()
    tokens = sz["batch"] * sz["seq"]
    out = {"table": "block", "sizes": sz, "tokens": tokens, "arms": {}}
    steps, warm = (3, 2) if small else (8, 3)
    for arm, swiglu, norm in (("moss", "fused", "fused"), ("bf16", "fused", "fused"), ("moss", "fused", "torch"), ("bf16", "fused", "torch"),
                              ("moss", "torch", "torch"), ("bf16", "torch", "torch")):
        b = blk.DecoderBlock(moss, torch, arm, swiglu=swiglu, norm=norm, **sz)
        for _ in range(warm):
            b.train_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            b.train_step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        key = arm + ("" if norm == "fused" else "_torch_norm") + ("" if swiglu == "fused" else "_torch_swiglu")
        out["arms"][key] = {"ms_per_step": round(ms, 3), "tokens_per_s": round(tokens / ms * 1e3, 1)}
        del b
        torch.cuda.empty_cache()
    out["speedup_moss_over_bf16"] = round(out["arms"]["bf16"]["ms_per_step"] / out["arms"]["moss"]["ms_per_step"], 3)
    out["linear_tflop_per_step"] = round(blk.linear_flops(sz["batch"], sz["seq"], sz["hidden"], sz["ffn"]) / 1e12, 3)
    out["attention_tflop_per_step"] = round(blk.attention_flops(sz["batch"], sz["seq"], sz["hidden"]) / 1e12, 3)
    out["note"] = ("bf16 arm: torch matmul (vendor BF16 GEMM) and torch fused AdamW; scaffolding identical in both arms (SwiGLU and "
                   "RMSNorm + residual add: the library's BF16 kernels, which in the moss arm also hand the tensor maxima to the "
                   "quantizers; *_torch_norm: torch rms_norm and add in both arms; *_torch_swiglu: torch silu and mul as well); "
                   "paper (8 x H800, full 7B model): 1.34x over BF16, context only")
    return out


def producer(moss, torch, small=False):
    """h = silu(gate) * up followed by the two-level quantization of h (both groupings) at the size of a
    LLaMA-7B feed-forward activation: torch's two elementwise kernels plus the searching quantizer against
    the library's SwiGLU, which leaves max|h| behind, plus the quantizer that takes it."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(45)
    rows, cols = (256, 512) if small else (8192, 11008)
    bf16 = torch.bfloat16
    g = (torch.randn((rows, cols), generator=gen, device=dev, dtype=torch.float32) * 2.0).to(bf16)
    u = torch.randn((rows, cols), generator=gen, device=dev, dtype=torch.float32).to(bf16)
    d = (torch.randn((rows, cols), generator=gen, device=dev, dtype=torch.float32) * 1e-3).to(bf16)
    both = moss.MOSS_Q_ROW | moss.MOSS_Q_COL
    u8 = torch.uint8
    out = dict(q_row=torch.empty((rows, cols), dtype=u8, device=dev), e_row=torch.empty((rows, cols // 32), dtype=u8, device=dev),
               q_col=torch.empty((cols, rows), dtype=u8, device=dev), e_col=torch.empty((cols, rows // 32), dtype=u8, device=dev),
               s=torch.empty(1, dtype=torch.float32, device=dev))
    ws = torch.empty(max(16, moss.load().moss_quant_workspace_bytes(rows, cols, both)), dtype=u8, device=dev)
    h = torch.empty_like(g)
    word = torch.empty(1, dtype=torch.int32, device=dev)
    dg, du = torch.empty_like(g), torch.empty_like(g)
    wg, wu = torch.empty(1, dtype=torch.int32, device=dev), torch.empty(1, dtype=torch.int32, device=dev)
    reps = 3 if small else 10
    n = rows * cols
    r = {}
    r["torch_silu_mul_ms"], _ = _time_ms(torch, lambda: torch.mul(torch.nn.functional.silu(g), u, out=h), reps)
    r["quant_searching_ms"], _ = _time_ms(torch, lambda: moss.quant_act_2level(h, both, out=out, workspace=ws), reps)
    r["swiglu_with_max_ms"], _ = _time_ms(torch, lambda: moss.swiglu_bf16(g, u, h=h, absmax_bits=word), reps)
    r["quant_given_max_ms"], _ = _time_ms(torch, lambda: moss.quant_act_2level_given_max(h, word, both, out=out), reps)
    r["swiglu_backward_with_max_ms"], _ = _time_ms(
        torch, lambda: moss.swiglu_bf16_backward(g, u, d, d_gate=dg, d_up=du, d_gate_absmax_bits=wg, d_up_absmax_bits=wu), reps)
    r = {k: round(v, 4) for k, v in r.items()}
    r["swiglu_gbs"] = round(n * 6.0 / (r["swiglu_with_max_ms"] * 1e-3) / 1e9, 1)                 # 2 x 2 B in, 2 B out
    r["swiglu_backward_gbs"] = round(n * 10.0 / (r["swiglu_backward_with_max_ms"] * 1e-3) / 1e9, 1)   # 3 x 2 B in, 2 x 2 B out
    r["quant_given_max_gbs"] = round(n * 4.0625 / (r["quant_given_max_ms"] * 1e-3) / 1e9, 1)
    r["chain_torch_then_search_ms"] = round(r["torch_silu_mul_ms"] + r["quant_searching_ms"], 4)
    r["chain_fused_ms"] = round(r["swiglu_with_max_ms"] + r["quant_given_max_ms"], 4)
    return {"table": "producer", "shape": [rows, cols], "unit": "ms", "times": r,
            "note": "torch_silu_mul: torch.nn.functional.silu then torch.mul (two elementwise kernels); the searching quantizer "
                    "reads h twice at this size (172 MiB), the one given the maximum once"}


def quant(moss, torch, small=False):
    """The activation quantizer alone (config 2 of the benchmark and the 7B activation widths): every call after a
    512 MiB fill that leaves the caches cold and full of dirty lines, timed between events; GB/s of the
    algorithmic bytes (2 B read + 1.03125 B written per element and grouping) and of the bytes actually moved
    (tensors above 64 MiB are read twice by the searching entry point).  For scale: a plain device copy of the
    same tensor (2 B read + 2 B written per element)."""
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(46)
    u8 = torch.uint8
    shapes = [(256, 512)] if small else [(8192, 4096), (8192, 11008), (8192, 12288)]
    flush = torch.empty((8 if small else 512) << 20, dtype=u8, device=dev)
    reps = 3 if small else 10
    rows_out = []

    def timed(fn):
        ts = []
        for i in range(reps + 2):
            flush.fill_(i & 0xFF)
            e0, e1 = _events(torch)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        ts = sorted(ts[2:])
        return ts[len(ts) // 2]
    for rows, cols in shapes:
        n = rows * cols
        x = (torch.randn((rows, cols), generator=gen, device=dev, dtype=torch.float32)).to(torch.bfloat16)
        out = dict(q_row=torch.empty((rows, cols), dtype=u8, device=dev), e_row=torch.empty((rows, cols // 32), dtype=u8, device=dev),
                   q_col=torch.empty((cols, rows), dtype=u8, device=dev), e_col=torch.empty((cols, rows // 32), dtype=u8, device=dev),
                   s=torch.empty(1, dtype=torch.float32, device=dev))
        ws = torch.empty(max(16, moss.load().moss_quant_workspace_bytes(rows, cols, 3)), dtype=u8, device=dev)
        ws_kept = torch.zeros_like(ws)         # zero-filled once, then only these calls write to it (MOSS_WS_KEPT)
        word = (x.view(torch.int16).to(torch.int32) & 0x7FFF).max().to(torch.int32).reshape(1)
        y = torch.empty_like(x)
        copy_ms = timed(lambda: y.copy_(x))
        for name, flags in (("row", moss.MOSS_Q_ROW), ("col", moss.MOSS_Q_COL), ("both", moss.MOSS_Q_ROW | moss.MOSS_Q_COL)):
            bpe = 2.0 + (2.0625 if name == "both" else 1.03125)
            twice = n * 2 > (64 << 20)
            ms = timed(lambda: moss.quant_act_2level(x, flags, out=out, workspace=ws))
            ms_kept = timed(lambda: moss.quant_act_2level(x, flags | moss.MOSS_WS_KEPT, out=out, workspace=ws_kept))
            ms_given = timed(lambda: moss.quant_act_2level_given_max(x, word, flags, out=out))
            rows_out.append({"rows": rows, "cols": cols, "groupings": name, "searching_ms": round(ms, 4),
                             "searching_kept_workspace_ms": round(ms_kept, 4),
                             "searching_algorithmic_gbs": round(n * bpe / ms / 1e6, 1),
                             "searching_moved_gbs": round(n * (bpe + (2.0 if twice else 0.0)) / ms / 1e6, 1),
                             "given_max_ms": round(ms_given, 4), "given_max_gbs": round(n * bpe / ms_given / 1e6, 1),
                             "device_copy_ms": round(copy_ms, 4), "device_copy_gbs": round(n * 4.0 / copy_ms / 1e6, 1)})
        del x, y, out
    return {"table": "quant", "unit": "ms", "rows": rows_out,
            "note": "event-bracketed single calls, each after a 512 MiB fill; the searching entry point is one launch up to 64 MiB "
                    "(X read once) and two launches above (X read twice); with a kept workspace the one-launch path drops its clearing launch"}


class _ClockPoller:
    """Samples the shader clock (the starred line of the driver's pp_dpm_sclk file) and the board power
    (hwmon power1_input) every two milliseconds while the GPU works."""

    def __init__(self):
        import glob
        import threading
        f = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        h = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*"))
        self._sclk_file = f[0] if f else None
        self._hwmon = h[0] if h else None
        self.sclk, self.power, self._stop = [], [], threading.Event()
        self._t = threading.Thread(target=self._run, daemon=True)

    def power_cap_w(self):
        try:
            return int(open(os.path.join(self._hwmon, "power1_cap")).read()) / 1e6
        except Exception:
            return None

    def _run(self):
        import re
        while not self._stop.is_set():
            try:
                if self._sclk_file:
                    m = re.search(r"(\d+)Mhz \*", open(self._sclk_file).read())
                    if m:
                        self.sclk.append(int(m.group(1)))
                if self._hwmon:
                    self.power.append(int(open(os.path.join(self._hwmon, "power1_input")).read()) / 1e6)
            except Exception:
                return
            self._stop.wait(0.002)

    def __enter__(self):
        self._t.start()
        return self

    def __exit__(self, *a):
        self._stop.set()
        self._t.join(timeout=15)

    @staticmethod
    def quantiles(v):
        v = sorted(v)
        return [v[int(q * (len(v) - 1))] for q in (0.1, 0.5, 0.9)] if v else None


def limits(moss, torch, small=False):
    """The same GEMM binary on operands of different content: the matrix cores draw more power the
    more operand bits toggle, and the clock follows.  Plus the bandwidth of a plain device copy as
    the practical ceiling of a read+write stream."""
    import time
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(44)
    M = N = K = 1024 if small else 8192
    secs = 0.3 if small else 3.0
    one = torch.ones(1, dtype=torch.float32, device=dev)
    out = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    ae = torch.full((M, K // 32), 127, dtype=torch.uint8, device=dev)
    x = torch.randn((M, K), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    w = (torch.randn((N, K), generator=gen, device=dev, dtype=torch.float32) * 0.02).to(torch.bfloat16)
    qx, qw = moss.quant_act_2level(x, moss.MOSS_Q_ROW), moss.quant_act_2level(w, moss.MOSS_Q_ROW)
    cases = [("constant codes (1.0)", torch.full((M, K), 0x38, dtype=torch.uint8, device=dev),
              torch.full((N, K), 0x38, dtype=torch.uint8, device=dev), ae),
             ("uniformly random codes", torch.randint(0, 120, (M, K), dtype=torch.uint8, device=dev, generator=gen),
              torch.randint(0, 120, (N, K), dtype=torch.uint8, device=dev, generator=gen), ae),
             ("quantized Gaussians", qx["q_row"], qw["q_row"], qx["e_row"])]
    rows, cap = [], None
    for name, a, b, e in cases:
        for _ in range(3):
            moss.gemm_fp8_mx(a, e, one, b, None, one, out=out)
        torch.cuda.synchronize()
        n = 0
        with _ClockPoller() as poll:
            t0 = time.time()
            while time.time() - t0 < secs:
                for _ in range(20):
                    moss.gemm_fp8_mx(a, e, one, b, None, one, out=out)
                torch.cuda.synchronize()
                n += 20
            dt = time.time() - t0
        rows.append({"operands": name, "us_per_gemm": round(dt / n * 1e6, 1), "tflops": round(2.0 * M * N * K * n / dt / 1e12, 1),
                     "sclk_mhz_p10_p50_p90": poll.quantiles(poll.sclk), "board_power_w_p10_p50_p90": poll.quantiles(poll.power),
                     "samples": len(poll.sclk)})
        cap = poll.power_cap_w()
    copies = []
    for mb in ([8] if small else [64, 1024]):
        src = torch.empty(mb << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        ms, _ = _time_ms(torch, lambda: dst.copy_(src), 10)
        copies.append({"mib": mb, "ms": round(ms, 4), "gbs_read_plus_write": round(2.0 * (mb << 20) / ms / 1e6, 1)})
    return {"table": "limits", "gemm_shape": [M, N, K], "board_power_cap_w": cap, "gemm_by_operand_content": rows, "device_copy": copies}


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("table", choices=["scaling", "gemm", "limits", "block", "producer", "quant"])
    ap.add_argument("--small", action="store_true", help="tiny shapes (used by the tests)")
    a = ap.parse_args(argv)
    import torch
    import paper_2511_05811_amd as moss
    if not torch.cuda.is_available():
        print("microbench needs the MI355X", file=sys.stderr)
        return 2
    res = {"scaling": scaling, "gemm": gemm, "limits": limits, "block": block, "producer": producer, "quant": quant}[a.table](moss, torch, a.small)
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
