#!/usr/bin/env python3
"""Benchmark of the MOSS FP8 hot path on one MI355X.

One "step" is one pass of the whole path over the five linears of a LLaMA-7B
decoder block at tokens = 8192 (batch 4 x seq 2048): for each linear
  forward : two-level quantization of X (row and column groupings in one call),
            Y = X W^T on the block-scaled FP8 matrix cores;
  backward: two-level quantization of dY (both groupings), dX = dY W, dW = dY^T X;
  update  : fused AdamW + automatic scale prediction + FP8 cast (+ transposed copy),
            fed with the dW the step just produced.
Inputs are the seeded synthetic tensors of moss_inputs.config3_linear (the ones the
parity tests check against the oracle), resident in HBM before the timed region.
The timed steps are then repeated with every library call bracketed by events on the
launch stream; the per-kernel-class figures of the `roofline` entries come from those.
Prints ONE JSON line on stdout.
"""
import argparse
import glob
import json
import os
import re
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP8_TFLOPS = 5000.0      # MI355X dense FP8 MFMA (published)
PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0
TOKENS = 8192
QUANT_BYTES_PER_ELEM_BOTH = 4.0625   # algorithmic: read 2 B, write 2 x (1 + 1/32) B
QUANT_ONE_LAUNCH_MAX_ELEMS = 8192 * 4096   # up to here X is read once; larger tensors are read twice (6.0625 B/elem moved)
WEIGHT_BYTES_PER_ELEM = 30.0         # W, m, v read+write (24) + FP32 grad (4) + codes (1) + transposed codes (1)
# Mean bytes per library call (all kernels of the call together; the GEMM is one launch) crossing the L2 boundary:
# FETCH_SIZE and WRITE_SIZE from two rocprofv3 --pmc runs of this script, each scaled by what the same counter
# reads for a plain copy (profiles/bench_config3_hbm_traffic.md).
TRAFFIC_BYTES_PER_LAUNCH = {"gemm": 7.00e8, "quant": 3.11e8, "weight": 1.215e9}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Workload:
    def __init__(self, dev, moss, torch):
        import numpy as np

        import moss_inputs as mi
        self.layers = []
        u8, f32, bf16 = torch.uint8, torch.float32, torch.bfloat16
        lib = moss.load()

        def up(bits):
            return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(bf16).to(dev)
        for index, (name, K, N) in enumerate(mi.LLAMA7B_LINEARS):
            xb, wb, dyb = mi.config3_linear(index, tokens=TOKENS)
            L = {"name": name, "K": K, "N": N}
            L["x"], L["dy"] = up(xb), up(dyb)
            L["w"] = torch.from_numpy(mi.bf16_bits_to_f32(wb)).to(dev)      # FP32 master weights
            del xb, wb, dyb
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
            L["ws_q"] = torch.zeros(max(16, lib.moss_quant_workspace_bytes(TOKENS, max(K, N), 3)), dtype=u8, device=dev)
            L["ws_w"] = torch.zeros(max(16, lib.moss_weight_workspace_bytes(N, K)), dtype=u8, device=dev)
            moss.weight_autoscale_init(L["w"], L["state"], wq=L["wq"], wq_t=L["wq_t"], workspace=L["ws_w"])
            L["s_w"] = L["state"][4:8].view(f32)
            self.layers.append(L)
        shapes = [(K, N) for _, K, N in mi.LLAMA7B_LINEARS]
        self.gemm_flops = sum(3 * 2.0 * TOKENS * K * N for K, N in shapes)
        self.quant_tensors = [TOKENS * K for K, _ in shapes] + [TOKENS * N for _, N in shapes]
        self.quant_elems = sum(self.quant_tensors)
        self.quant_moved_bytes = sum(n * (QUANT_BYTES_PER_ELEM_BOTH + (2.0 if n > QUANT_ONE_LAUNCH_MAX_ELEMS else 0.0))
                                     for n in self.quant_tensors)
        self.weight_elems = sum(K * N for K, N in shapes)


def adamw_args(moss, t):
    import numpy as np
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.95))
    return moss.AdamWArgs(3e-4, 0.9, 0.95, 1e-8, 0.1, 1.0 - b1, 1.0 - b2, 1.0 - b1 ** t, 1.0 - b2 ** t, 1.0, 500, t)


def run_step(wl, moss, torch, t, rec):
    """One pass of the whole path.  rec(kind) returns a context that brackets a call with events."""
    both = moss.MOSS_Q_ROW | moss.MOSS_Q_COL | moss.MOSS_WS_KEPT      # (ws_q: zero-filled above, used by these calls only)
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


class ClockPoller:
    """Samples the shader clock (the starred line of the driver's pp_dpm_sclk file) and the board power
    about once a millisecond while the GPU works: the block-scaled GEMM lowers the clock on realistic
    operands, and a roofline fraction against the nominal 2.4 GHz peak should say at which clock it ran."""

    def __init__(self):
        self.sclk, self.power = [], []
        self._stop = threading.Event()
        f = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        p = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        self._sclk_file = f[0] if f else None
        self._power_file = p[0] if p else None
        self._t = threading.Thread(target=self._run, daemon=True)

    def _run(self):
        while not self._stop.is_set():
            try:
                if self._sclk_file:
                    m = re.search(r"(\d+)Mhz \*", open(self._sclk_file).read())
                    if m:
                        self.sclk.append(int(m.group(1)))
                if self._power_file:
                    self.power.append(int(open(self._power_file).read()) / 1e6)
            except Exception:
                return
            self._stop.wait(0.001)

    def __enter__(self):
        self._t.start()
        return self

    def __exit__(self, *a):
        self._stop.set()
        self._t.join(timeout=5)

    def summary(self):
        def med(v):
            v = sorted(v)
            return v[len(v) // 2] if v else None
        return {"sclk_mhz_median": med(self.sclk), "sclk_mhz_min": min(self.sclk) if self.sclk else None,
                "sclk_mhz_max": max(self.sclk) if self.sclk else None, "power_w_median": med(self.power),
                "samples": len(self.sclk)}


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
    ap.add_argument("--no-side-baselines", action="store_true", help="skip the BF16 GEMM comparison runs")
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

    # timed region: exactly `steps` passes, wall clock bracketed by synchronizations (the shader clock is sampled
    # from the driver's files meanwhile)
    with ClockPoller() as clocks:
        t0 = time.perf_counter()
        for _ in range(args.steps):
            t += 1
            run_step(wl, moss, torch, t, off)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3

    # the same steps again with every call bracketed by events on the launch stream: per-kernel-class durations
    # (the events themselves cost about 2 % of a step, which is why they stay out of the timed region)
    rec = Recorder(torch, True)
    for _ in range(args.steps):
        t += 1
        run_step(wl, moss, torch, t, rec)
    torch.cuda.synchronize()
    tot, cnt = rec.totals_ms(), rec.counts()
    per_step = {k: tot[k] / args.steps for k in tot}
    launches = {k: cnt[k] // args.steps for k in cnt}

    gemm_tflops = wl.gemm_flops / (per_step["gemm"] * 1e-3) / 1e12
    quant_gbs = wl.quant_elems * QUANT_BYTES_PER_ELEM_BOTH / (per_step["quant"] * 1e-3) / 1e9
    quant_moved_gbs = wl.quant_moved_bytes / (per_step["quant"] * 1e-3) / 1e9
    weight_gbs = wl.weight_elems * WEIGHT_BYTES_PER_ELEM / (per_step["weight"] * 1e-3) / 1e9

    def entry(kind, bound, kernel, achieved, peak, unit, **extra):
        e = {"bound": bound, "kernel": kernel, "achieved": round(achieved, 2), "peak": peak, "unit": unit,
             "frac": round(achieved / peak, 4), "avg_call_ms": round(per_step[kind] / launches[kind], 4),
             "calls_per_step": launches[kind], "ms_per_step": round(per_step[kind], 4),
             "traffic": TRAFFIC_BYTES_PER_LAUNCH[kind]}
        e.update(extra)
        return e
    rooflines = {
        "gemm_fp8_mx": entry("gemm", "mfma", "k_gemm_mx_big (moss_gemm_fp8_mx)", gemm_tflops, PEAK_FP8_TFLOPS, "TFLOP/s",
                             algorithmic="2 M N K per launch", clocks_in_timed_region=clocks.summary(),
                             traffic_note="bytes per launch crossing the L2 boundary; the operand re-fetches of the 8 L2s are "
                                          "served by the Infinity Cache"),
        "quant_act_2level": entry("quant", "hbm", "k_quant_persist (<= 64 MiB) / k_amax_bf16 + k_quant_tile", quant_gbs,
                                  PEAK_HBM_GBS, "GB/s", algorithmic=f"{QUANT_BYTES_PER_ELEM_BOTH} B/element (both groupings)",
                                  moved_gbs=round(quant_moved_gbs, 1),
                                  moved_note="tensors above 64 MiB are read twice (6.0625 B/element moved)"),
        "weight_autoscale_cast": entry("weight", "hbm", "k_weight_tile (moss_weight_autoscale_cast)", weight_gbs, PEAK_HBM_GBS,
                                       "GB/s", algorithmic=f"{WEIGHT_BYTES_PER_ELEM} B/element"),
    }

    value = wl.gemm_flops / (ms_per_step * 1e-3) / 1e12
    dominant = dict(rooflines["gemm_fp8_mx"])
    dominant["avg_launch_ms"] = dominant["avg_call_ms"]
    dominant["launches_per_step"] = dominant["calls_per_step"]
    result = {
        "metric": "MOSS FP8 linear fwd+bwd+update, GEMM TFLOP/s over the whole hot-path step (7B linear shapes)",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8_e4m3 (fp32 accumulate)", "data": "synthetic",
        "config": {"workload": "configs[2]: LLaMA-7B linears (qkv, o, gate, up, down) fwd+bwd at tokens=8192, "
                               "two-level quantizers + fused AdamW/autoscale cast + block-scaled FP8 GEMMs",
                   "tokens": TOKENS, "gemm_tflop_per_step": round(wl.gemm_flops / 1e12, 3)},
        "roofline": dominant,
        "rooflines": rooflines,
    }

    if not args.no_side_baselines:
        # BF16 hand GEMM baseline on the same 15 GEMM shapes (reported, not part of the step)
        def bf16_pass(fn):
            ms = 0.0
            for L in wl.layers:
                K, N = L["K"], L["N"]
                wb = L["w"].to(torch.bfloat16); wbt = wb.t().contiguous()
                xt = L["x"].t().contiguous(); dyt = L["dy"].t().contiguous()
                for a, b, o in ((L["x"], wb, L["y"]), (L["dy"], wbt, L["dx"]),
                                (dyt, xt, torch.empty((N, K), dtype=torch.bfloat16, device=dev))):
                    fn(a, b, o)
                    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
                    e0.record()
                    fn(a, b, o)
                    e1.record(); torch.cuda.synchronize()
                    ms += e0.elapsed_time(e1)
            return ms
        bf_ms = bf16_pass(lambda a, b, o: moss.gemm_bf16_baseline(a, b, out=o))
        bv_ms = bf16_pass(lambda a, b, o: torch.matmul(a, b.t(), out=o))
        result["side_baselines"] = {
            "gemm_bf16_hand": {"ms_for_same_gemms": round(bf_ms, 4), "tflops": round(wl.gemm_flops / bf_ms / 1e9, 2),
                               "frac_of_bf16_peak": round(wl.gemm_flops / bf_ms / 1e9 / PEAK_BF16_TFLOPS, 4)},
            "gemm_bf16_vendor": {"ms_for_same_gemms": round(bv_ms, 4), "tflops": round(wl.gemm_flops / bv_ms / 1e9, 2),
                                 "frac_of_bf16_peak": round(wl.gemm_flops / bv_ms / 1e9 / PEAK_BF16_TFLOPS, 4),
                                 "note": "torch.matmul on BF16 copies of the same operands"}}
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
