#!/usr/bin/env python3
"""Benchmark of the MOSS FP8 hot path on one MI355X.

One "step" is one pass of the whole path over the five linears of a LLaMA-7B
decoder block at tokens = 8192 (batch 4 x seq 2048): for each linear
  forward : two-level quantization of X (row and column groupings in one call),
            Y = X W^T on the block-scaled FP8 matrix cores;
  backward: two-level quantization of dY (both groupings), dX = dY W, dW = dY^T X;
  update  : fused AdamW + automatic scale prediction + FP8 cast (+ transposed copy),
            fed with the dW the step just produced.
Inputs are synthetic (seeded torch generators on the device) and resident in HBM
before the timed region.  Prints ONE JSON line on stdout.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP8_TFLOPS = 5000.0      # MI355X dense FP8 MFMA (published)
PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
TOKENS = 8192
LINEARS = [("qkv", 4096, 12288), ("o", 4096, 4096), ("gate", 4096, 11008), ("up", 4096, 11008), ("down", 11008, 4096)]
QUANT_BYTES_PER_ELEM_BOTH = 4.0625   # read 2 B, write 2 x (1 + 1/32) B
WEIGHT_BYTES_PER_ELEM = 30.0         # W, m, v read+write (24) + FP32 grad (4) + codes (1) + transposed codes (1)
# Mean bytes per GEMM launch crossing the L2 boundary (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000 from two
# rocprofv3 --pmc runs of this script; summary and scale factors in profiles/bench_config3_hbm_traffic.md).
GEMM_TRAFFIC_BYTES_PER_LAUNCH = 6.98e8


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Workload:
    def __init__(self, dev, moss, torch):
        gen = torch.Generator(device=dev)
        gen.manual_seed(3)
        self.layers = []
        u8, f32, bf16 = torch.uint8, torch.float32, torch.bfloat16
        for name, K, N in LINEARS:
            L = {"name": name, "K": K, "N": N}
            L["x"] = torch.randn((TOKENS, K), generator=gen, device=dev, dtype=f32).to(bf16)
            L["dy"] = (torch.randn((TOKENS, N), generator=gen, device=dev, dtype=f32) * 1e-3).to(bf16)
            L["w"] = torch.randn((N, K), generator=gen, device=dev, dtype=f32) * 0.02
            L["m"] = torch.zeros_like(L["w"]); L["v"] = torch.zeros_like(L["w"])
            L["state"] = moss.new_wscale_state(dev)
            L["wq"] = torch.empty((N, K), dtype=u8, device=dev)
            L["wq_t"] = torch.empty((K, N), dtype=u8, device=dev)
            for key, (r, c) in (("qx", (TOKENS, K)), ("qdy", (TOKENS, N))):
                L[key] = dict(q_row=torch.empty((r, c), dtype=u8, device=dev), e_row=torch.empty((r, c // 32), dtype=u8, device=dev),
                              q_col=torch.empty((c, r), dtype=u8, device=dev), e_col=torch.empty((c, r // 32), dtype=u8, device=dev),
                              s=torch.empty(1, dtype=f32, device=dev))
            L["y"] = torch.empty((TOKENS, N), dtype=bf16, device=dev)
            L["dx"] = torch.empty((TOKENS, K), dtype=bf16, device=dev)
            L["dw"] = torch.empty((N, K), dtype=f32, device=dev)
            lib = moss.load()
            L["ws_q"] = torch.empty(max(16, lib.moss_quant_workspace_bytes(TOKENS, max(K, N), 3)), dtype=u8, device=dev)
            L["ws_w"] = torch.empty(max(16, lib.moss_weight_workspace_bytes(N, K)), dtype=u8, device=dev)
            moss.weight_autoscale_init(L["w"], L["state"], wq=L["wq"], wq_t=L["wq_t"], workspace=L["ws_w"])
            L["s_w"] = L["state"][4:8].view(f32)
            self.layers.append(L)
        self.gemm_flops = sum(3 * 2.0 * TOKENS * K * N for _, K, N in LINEARS)
        self.quant_elems = sum(TOKENS * (K + N) for _, K, N in LINEARS)
        self.weight_elems = sum(K * N for _, K, N in LINEARS)


def adamw_args(moss, t):
    import numpy as np
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.95))
    return moss.AdamWArgs(3e-4, 0.9, 0.95, 1e-8, 0.1, 1.0 - b1, 1.0 - b2, 1.0 - b1 ** t, 1.0 - b2 ** t, 1.0, 500, t)


def run_step(wl, moss, torch, t, rec=None):
    """One pass of the whole path.  rec(kind) returns a context that brackets a call with events."""
    both = moss.MOSS_Q_ROW | moss.MOSS_Q_COL
    f32 = torch.float32
    for L in wl.layers:
        with rec("quant"):
            moss.quant_act_2level(L["x"], both, out=L["qx"], workspace=L["ws_q"])
        with rec("gemm"):
            moss.gemm_fp8_mx(L["qx"]["q_row"], L["qx"]["e_row"], L["qx"]["s"], L["wq"], None, L["s_w"], out=L["y"])
        with rec("quant"):
            moss.quant_act_2level(L["dy"], both, out=L["qdy"], workspace=L["ws_q"])
        with rec("gemm"):
            moss.gemm_fp8_mx(L["qdy"]["q_row"], L["qdy"]["e_row"], L["qdy"]["s"], L["wq_t"], None, L["s_w"], out=L["dx"])
        with rec("gemm"):
            moss.gemm_fp8_mx(L["qdy"]["q_col"], L["qdy"]["e_col"], L["qdy"]["s"], L["qx"]["q_col"], L["qx"]["e_col"],
                             L["qx"]["s"], out=L["dw"], out_dtype=f32)
        with rec("weight"):
            moss.weight_autoscale_cast(L["w"], L["m"], L["v"], L["dw"], adamw_args(moss, t), L["state"],
                                       wq=L["wq"], wq_t=L["wq_t"], workspace=L["ws_w"])


class Recorder:
    """Brackets calls with events on torch's current stream (the stream the binding launches on)."""

    def __init__(self, torch, enabled):
        self.torch, self.enabled, self.items = torch, enabled, []

    def __call__(self, kind):
        return _Span(self, kind)

    def totals_ms(self):
        out = {}
        for kind, a, b in self.items:
            out[kind] = out.get(kind, 0.0) + a.elapsed_time(b)
        return out

    def counts(self):
        out = {}
        for kind, _, _ in self.items:
            out[kind] = out.get(kind, 0) + 1
        return out


class _Span:
    def __init__(self, rec, kind):
        self.rec, self.kind = rec, kind

    def __enter__(self):
        if self.rec.enabled:
            self.a = self.rec.torch.cuda.Event(enable_timing=True)
            self.b = self.rec.torch.cuda.Event(enable_timing=True)
            self.a.record()

    def __exit__(self, *exc):
        if self.rec.enabled:
            self.b.record()
            self.rec.items.append((self.kind, self.a, self.b))
        return False


def cpu_baseline():
    """The CPU oracle, as it stands, timed on the host cores on a bounded sample of the same
    path: the 4096 -> 4096 linear at tokens = 192 (quantizers, weight step, three GEMMs)."""
    import numpy as np

    import moss_inputs as mi
    from oracle import moss_oracle as oracle
    tokens, K, N = 192, 4096, 4096
    xb, wb, dyb = mi.config3_linear(1, tokens=tokens)
    w = mi.bf16_bits_to_f32(wb).copy(); m = np.zeros_like(w); v = np.zeros_like(w)
    st, wq, wq_t = oracle.weight_init(w, want_transpose=True)
    t0 = time.perf_counter()
    qxr = oracle.quant_act_2level(xb, 0, 0); qxc = oracle.quant_act_2level(xb, 1, 0)
    y = oracle.gemm(qxr[0], qxr[1], qxr[2], wq, None, st.s_cur)
    qdr = oracle.quant_act_2level(dyb, 0, 0); qdc = oracle.quant_act_2level(dyb, 1, 0)
    dx = oracle.gemm(qdr[0], qdr[1], qdr[2], wq_t, None, st.s_cur)
    dw = oracle.gemm(qdc[0], qdc[1], qdc[2], qxc[0], qxc[1], qxc[2])
    hp = mi.adamw_hparams(1)
    oracle.weight_step(w, m, v, dw.astype(np.float32), oracle.adamw_args(**hp), st, want_transpose=True)
    dt = time.perf_counter() - t0
    flops = 3 * 2.0 * tokens * K * N
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"one 4096->4096 linear fwd+bwd+update at tokens={tokens} (full path, FP64 GEMM), {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the measurement run one plain 256 MiB device copy (a kernel of known traffic "
                         "against which hardware byte counters can be scaled)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py measures one GPU only: this build has no multi-GPU path; run it with --gpus 1.")
        sys.exit(2)

    import torch

    import paper_2511_05811_amd as moss
    moss.load()                      # fails loudly if the HIP library is not built
    if not torch.cuda.is_available():
        log("no GPU visible")
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = Workload(dev, moss, torch)
    torch.cuda.synchronize()

    t = 0
    off = Recorder(torch, False)
    for _ in range(args.warmup):
        t += 1
        run_step(wl, moss, torch, t, off)
    torch.cuda.synchronize()

    # timed region: exactly `steps` passes, wall clock bracketed by synchronizations
    t0 = time.perf_counter()
    for _ in range(args.steps):
        t += 1
        run_step(wl, moss, torch, t, off)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3

    # the same steps again with every call bracketed by events: per-kernel-class durations
    rec = Recorder(torch, True)
    for _ in range(args.steps):
        t += 1
        run_step(wl, moss, torch, t, rec)
    torch.cuda.synchronize()
    tot, cnt = rec.totals_ms(), rec.counts()
    gemm_ms = tot["gemm"] / args.steps
    quant_ms = tot["quant"] / args.steps
    weight_ms = tot["weight"] / args.steps
    gemm_tflops = wl.gemm_flops / (gemm_ms * 1e-3) / 1e12
    quant_gbs = wl.quant_elems * QUANT_BYTES_PER_ELEM_BOTH / (quant_ms * 1e-3) / 1e9
    weight_gbs = wl.weight_elems * WEIGHT_BYTES_PER_ELEM / (weight_ms * 1e-3) / 1e9

    # BF16 hand GEMM baseline on the same 15 GEMM shapes (reported, not part of the step)
    bf_ms = 0.0
    for L in wl.layers:
        K, N = L["K"], L["N"]
        wb = L["w"].to(torch.bfloat16); wbt = wb.t().contiguous()
        xt = L["x"].t().contiguous(); dyt = L["dy"].t().contiguous()
        for a, b, o in ((L["x"], wb, L["y"]), (L["dy"], wbt, L["dx"]), (dyt, xt, torch.empty((N, K), dtype=torch.bfloat16, device=dev))):
            moss.gemm_bf16_baseline(a, b, out=o)
            e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            moss.gemm_bf16_baseline(a, b, out=o)
            e1.record(); torch.cuda.synchronize()
            bf_ms += e0.elapsed_time(e1)
    bf16_tflops = wl.gemm_flops / (bf_ms * 1e-3) / 1e12
    # ... and on the vendor library's BF16 GEMM (torch.matmul), for scale
    bv_ms = 0.0
    for L in wl.layers:
        K, N = L["K"], L["N"]
        wb = L["w"].to(torch.bfloat16); wbt = wb.t().contiguous()
        xt = L["x"].t().contiguous(); dyt = L["dy"].t().contiguous()
        for a, b, o in ((L["x"], wb, L["y"]), (L["dy"], wbt, L["dx"]), (dyt, xt, torch.empty((N, K), dtype=torch.bfloat16, device=dev))):
            torch.matmul(a, b.t(), out=o)
            e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
            e0.record()
            torch.matmul(a, b.t(), out=o)
            e1.record(); torch.cuda.synchronize()
            bv_ms += e0.elapsed_time(e1)
    bf16_vendor_tflops = wl.gemm_flops / (bv_ms * 1e-3) / 1e12

    value = wl.gemm_flops / (ms_per_step * 1e-3) / 1e12
    result = {
        "metric": "MOSS FP8 linear fwd+bwd+update, GEMM TFLOP/s over the whole hot-path step (7B linear shapes)",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8_e4m3 (fp32 accumulate)", "data": "synthetic",
        "config": {"workload": "configs[2]: LLaMA-7B linears (qkv, o, gate, up, down) fwd+bwd at tokens=8192, "
                               "two-level quantizers + fused AdamW/autoscale cast + block-scaled FP8 GEMMs",
                   "tokens": TOKENS, "gemm_tflop_per_step": round(wl.gemm_flops / 1e12, 3)},
        "roofline": {"bound": "mfma", "kernel": "k_gemm (moss_gemm_fp8_mx)", "achieved": round(gemm_tflops, 2),
                     "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s", "frac": round(gemm_tflops / PEAK_FP8_TFLOPS, 4),
                     "avg_launch_ms": round(gemm_ms / (cnt["gemm"] / args.steps), 4),
                     "launches_per_step": cnt["gemm"] // args.steps, "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH,
                     "traffic_note": "bytes per launch leaving/entering the L2 (rocprofv3 FETCH_SIZE/WRITE_SIZE, scaled "
                                     "against a plain copy); the operand re-fetches are served by the Infinity Cache"},
        "components": {
            "gemm_fp8": {"ms_per_step": round(gemm_ms, 4), "tflops": round(gemm_tflops, 2),
                         "frac_of_fp8_peak": round(gemm_tflops / PEAK_FP8_TFLOPS, 4)},
            "quant_act_2level": {"ms_per_step": round(quant_ms, 4), "gbs": round(quant_gbs, 1),
                                 "frac_of_hbm_peak": round(quant_gbs / PEAK_HBM_GBS, 4),
                                 "bytes_per_elem": QUANT_BYTES_PER_ELEM_BOTH},
            "weight_autoscale_cast": {"ms_per_step": round(weight_ms, 4), "gbs": round(weight_gbs, 1),
                                      "frac_of_hbm_peak": round(weight_gbs / PEAK_HBM_GBS, 4),
                                      "bytes_per_elem": WEIGHT_BYTES_PER_ELEM},
            "gemm_bf16_baseline": {"ms_for_same_gemms": round(bf_ms, 4), "tflops": round(bf16_tflops, 2),
                                   "frac_of_bf16_peak": round(bf16_tflops / PEAK_BF16_TFLOPS, 4)},
            "gemm_bf16_vendor": {"ms_for_same_gemms": round(bv_ms, 4), "tflops": round(bf16_vendor_tflops, 2),
                                 "frac_of_bf16_peak": round(bf16_vendor_tflops / PEAK_BF16_TFLOPS, 4),
                                 "note": "torch.matmul on BF16 copies of the same operands"},
        },
    }
    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        try:
            result["cpu_baseline"] = cpu_baseline()
        except Exception as exc:   # the GPU numbers stand on their own
            result["cpu_baseline"] = {"error": repr(exc)}
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
