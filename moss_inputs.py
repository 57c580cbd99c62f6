"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke run.

This module only draws random numbers and converts storage formats.  It holds
none of the method's arithmetic (no scales, no FP8 rounding, no optimizer
math) and imports neither the HIP binding nor the CPU oracle.

The workloads stand in for the paper's LLaMA/OLMo-7B tensors (hidden 4096,
FFN 11008, 32 heads; appendix table of model sizes): same shapes, heavy-tailed
values with a few outlier channels as motivated in the paper's introduction.
"""
import numpy as np

# (K, N) of the five linears of one 7B decoder block: QKV, O, gate, up, down.
LLAMA7B_LINEARS = [("qkv", 4096, 12288), ("o", 4096, 4096), ("gate", 4096, 11008),
                   ("up", 4096, 11008), ("down", 11008, 4096)]
TOKENS_7B = 8192


def f32_to_bf16_bits(a):
    """Round-to-nearest-even conversion of finite float32 values to BF16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def config1(seed=1):
    """Single linear forward: X [256x1024] ~ N(0,1) with 8 outlier channels x50, W [1024x1024] ~ N(0,0.02)."""
    rng = _rng(seed)
    x = rng.standard_normal((256, 1024), dtype=np.float32)
    cols = rng.choice(1024, 8, replace=False)
    x[:, cols] *= 50.0
    w = rng.standard_normal((1024, 1024), dtype=np.float32) * np.float32(0.02)
    return f32_to_bf16_bits(x), f32_to_bf16_bits(w)


def heavy_tailed_activation(rows, cols, seed=2, outlier_frac=0.01, outlier_gain=100.0, return_channels=False):
    """0.5 * Student-t(nu=3) with a fraction of the channels multiplied by a gain (BF16 bits);
    with return_channels also the indices of those channels."""
    rng = _rng(seed)
    x = (0.5 * rng.standard_t(3.0, size=(rows, cols))).astype(np.float32)
    n_out = max(1, int(round(outlier_frac * cols)))
    ch = rng.choice(cols, n_out, replace=False)
    x[:, ch] *= np.float32(outlier_gain)
    return (f32_to_bf16_bits(x), np.sort(ch)) if return_channels else f32_to_bf16_bits(x)


def config2(seed=2, rows=8192, cols=4096):
    """Activation quantizer at 7B scale."""
    return heavy_tailed_activation(rows, cols, seed)


def config3_linear(index, tokens=TOKENS_7B, seed=3, k=None, n=None):
    """Operands of linear `index` of LLAMA7B_LINEARS (or an explicit k, n):
    X [tokens x K] ~ N(0,1), W [N x K] ~ N(0,0.02), dY [tokens x N] ~ N(0,1e-3); all BF16 bits."""
    if k is None:
        _, k, n = LLAMA7B_LINEARS[index]
    rng = _rng(seed + index)
    x = rng.standard_normal((tokens, k), dtype=np.float32)
    w = rng.standard_normal((n, k), dtype=np.float32) * np.float32(0.02)
    dy = rng.standard_normal((tokens, n), dtype=np.float32) * np.float32(1e-3)
    return f32_to_bf16_bits(x), f32_to_bf16_bits(w), f32_to_bf16_bits(dy)


def config4_weights(rows=4096, cols=11008, seed=4):
    """FP32 master weights ~ N(0, 0.02)."""
    return _rng(seed).standard_normal((rows, cols), dtype=np.float32) * np.float32(0.02)


def config4_is_spike_step(t):
    """Deterministic 5% of the steps carry a x20 gradient spike."""
    return ((t * 2654435761) % (1 << 32)) < int(0.05 * (1 << 32))


def config4_grad(t, rows=4096, cols=11008, seed=4, sparse_spikes=False):
    """Synthetic gradient of step t (1-based) ~ N(0,1e-3); whole-tensor x20 on spike
    steps, or (sparse_spikes) 0.1% of the elements x20 on every step."""
    rng = _rng(seed * 1000003 + t)
    g = rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(1e-3)
    if sparse_spikes:
        mask = rng.random((rows, cols), dtype=np.float32) < np.float32(1e-3)
        g[mask] *= np.float32(20.0)
    elif config4_is_spike_step(t):
        g *= np.float32(20.0)
    return g


def adamw_hparams(step, lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1,
                  margin=1.0, interval=500):
    """Plain numbers for optimizer step `step` (1-based).  The (1-beta) and bias
    correction terms are formed in double from the single-precision betas and are
    rounded to single by whoever stores them; both implementations receive them
    as inputs."""
    b1 = float(np.float32(beta1))
    b2 = float(np.float32(beta2))
    return dict(lr=lr, beta1=beta1, beta2=beta2, eps=eps, weight_decay=weight_decay,
                one_minus_beta1=1.0 - b1, one_minus_beta2=1.0 - b2,
                bias_corr1=1.0 - b1 ** step, bias_corr2=1.0 - b2 ** step,
                margin=margin, interval=interval)


def adversarial_activations(rows=64, cols=128, seed=7):
    """Edge-case activation tensors (BF16 bits) keyed by name."""
    rng = _rng(seed)
    base = rng.standard_normal((rows, cols), dtype=np.float32)
    out = {}
    out["zeros"] = np.zeros((rows, cols), np.float32)
    z = base.copy(); z[:, 32:64] = 0.0; z[5, :] = 0.0
    out["zero_groups"] = z
    o = base.copy(); o[3, 17] = 3.0e4
    out["one_outlier"] = o
    sgn = base.copy(); sgn[::2, ::3] = -0.0; sgn[1::2, ::5] = 0.0
    out["signed_zeros"] = sgn
    tiny = base * np.float32(2.0 ** -120)
    out["tiny"] = tiny
    tz = tiny.copy(); tz[:, 64:96] = 0.0; tz[7, :] = -0.0
    out["tiny_zero_groups"] = tz
    out["subnormal"] = base * np.float32(2.0 ** -127)      # BF16 subnormals, 1/s beyond FP32 range
    mixed = base.copy(); mixed[:, 0:32] *= np.float32(2.0 ** -125); mixed[9, 40] = 200.0
    out["tiny_groups_under_large_max"] = mixed
    big = base * np.float32(2.0 ** 90)
    out["big"] = big
    # group maxima placed on both sides of sqrt(2) * 2^k relative to the tensor maximum
    sq = np.full((rows, cols), 0.01, np.float32)
    sq[0, 0] = 1.0
    ratios = [1.40625, 1.4140625, 1.421875, 0.70703125, 0.703125, 0.7109375, 1.0, 0.5, 0.25, 0.35546875]
    for i, r in enumerate(ratios):
        sq[1 + i, (i % (cols // 32)) * 32 + 3] = np.float32(r) * np.float32(2.0 ** -(i % 5))
    out["sqrt2_boundary"] = sq
    w = np.exp(rng.uniform(-40, 10, size=(rows, cols))).astype(np.float32) * np.sign(base)
    out["wide_range"] = w
    return {k: f32_to_bf16_bits(v) for k, v in out.items()}
