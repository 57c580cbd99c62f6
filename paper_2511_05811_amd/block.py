"""One LLaMA-style decoder block training step with its linears on the MOSS FP8 path.

This is measurement scaffolding around the library, not part of it: RMSNorm, rotary embedding,
causal attention, SwiGLU and the residual adds are ordinary BF16 torch operations, identical in
both arms of the comparison, exactly as the paper leaves them in BF16 (Sec. 4.1).  Only the
linear layers differ:

  arm "moss": X and dY are two-level quantized (both groupings in one call), the three GEMMs
              run on the block-scaled FP8 matrix cores, the optimizer step is the fused
              AdamW + automatic scaling + FP8 cast of the library;
  arm "bf16": the same three GEMMs as BF16 torch matmuls, AdamW as torch's fused optimizer on
              FP32 master weights followed by a BF16 copy.

Q, K and V are one fused hidden -> 3 hidden linear; gate and up are separate linears.

SwiGLU and RMSNorm (the second one fused with the residual add in front of it, its backward with the
gradient of the residual path) are the library's BF16 kernels in both arms (`swiglu="fused"`,
`norm="fused"`, the defaults) or torch's operations (`"torch"`).  In the "moss" arm the fused kernels
also hand the maximum of what they wrote to the quantizer of the linear that consumes it, which
then needs no search pass: the inputs of all five linears but the attention output, and every
dY but that of the QKV projection (it comes out of torch's attention backward) and of the down
projection (the upstream gradient).
"""


class _MaxWords:
    """Side channel from a producer to the quantizers of the tensor it wrote: the device word that holds the
    tensor's maximum, keyed by the tensor's storage.  A word stays valid for every consumer of the tensor (the
    normalised hidden state feeds two projections) as long as nothing has written to the tensor since: its
    version counter is part of the entry."""

    def __init__(self):
        self.words = {}
        self.used = 0

    def put(self, tensor, word):
        self.words[tensor.data_ptr()] = (tuple(tensor.shape), tensor._version, word)

    def take(self, tensor):
        e = self.words.get(tensor.data_ptr())
        if e is None or e[0] != tuple(tensor.shape) or e[1] != tensor._version:
            return None
        self.used += 1
        return e[2]

    def clear(self):
        self.words.clear()
def _adamw_args(moss, t, lr=3e-4, interval=500):
    import numpy as np
    b1, b2 = float(np.float32(0.9)), float(np.float32(0.95))
    return moss.AdamWArgs(lr, 0.9, 0.95, 1e-8, 0.1, 1.0 - b1, 1.0 - b2, 1.0 - b1 ** t, 1.0 - b2 ** t, 1.0, interval, t)


class _MossLinear:
    """FP32 master weight [N x K] with its FP8 copies, optimizer state and per-layer buffers."""

    def __init__(self, moss, torch, tokens, k, n, gen, dev, words=None):
        u8, f32 = torch.uint8, torch.float32
        self.moss, self.k, self.n, self.words = moss, k, n, words
        self.w = torch.randn((n, k), generator=gen, device=dev, dtype=f32) * 0.02
        self.m = torch.zeros_like(self.w)
        self.v = torch.zeros_like(self.w)
        self.dw = torch.empty((n, k), dtype=f32, device=dev)
        self.state = moss.new_wscale_state(dev)
        self.wq = torch.empty((n, k), dtype=u8, device=dev)
        self.wq_t = torch.empty((k, n), dtype=u8, device=dev)
        lib = moss.load()
        self.ws_w = torch.empty(max(16, lib.moss_weight_workspace_bytes(n, k)), dtype=u8, device=dev)
        self.ws_q = torch.zeros(max(16, lib.moss_quant_workspace_bytes(tokens, max(k, n), 3)), dtype=u8, device=dev)
        moss.weight_autoscale_init(self.w, self.state, wq=self.wq, wq_t=self.wq_t, workspace=self.ws_w)
        self.s_w = self.state[4:8].view(f32)

        def qbuf(r, c):
            return dict(q_row=torch.empty((r, c), dtype=u8, device=dev), e_row=torch.empty((r, c // 32), dtype=u8, device=dev),
                        q_col=torch.empty((c, r), dtype=u8, device=dev), e_col=torch.empty((c, r // 32), dtype=u8, device=dev),
                        s=torch.empty(1, dtype=f32, device=dev))
        self.qx, self.qdy = qbuf(tokens, k), qbuf(tokens, n)

    def step(self, t):
        self.moss.weight_autoscale_cast(self.w, self.m, self.v, self.dw, _adamw_args(self.moss, t), self.state,
                                        wq=self.wq, wq_t=self.wq_t, workspace=self.ws_w)


def _moss_linear_fn(torch):
    class Fn(torch.autograd.Function):
        @staticmethod
        def forward(ctx, x, layer):
            moss = layer.moss
            both = moss.MOSS_Q_ROW | moss.MOSS_Q_COL
            x = x.contiguous()
            word = layer.words.take(x) if layer.words is not None else None
            if word is not None:
                moss.quant_act_2level_given_max(x, word, both, out=layer.qx)
            else:
                moss.quant_act_2level(x, both | moss.MOSS_WS_KEPT, out=layer.qx, workspace=layer.ws_q)
            ctx.layer = layer
            return moss.gemm_fp8_mx(layer.qx["q_row"], layer.qx["e_row"], layer.qx["s"], layer.wq, None, layer.s_w)

        @staticmethod
        def backward(ctx, dy):
            layer = ctx.layer
            moss = layer.moss
            both = moss.MOSS_Q_ROW | moss.MOSS_Q_COL
            dy = dy.contiguous()
            word = layer.words.take(dy) if layer.words is not None else None
            if word is not None:
                moss.quant_act_2level_given_max(dy, word, both, out=layer.qdy)
            else:
                moss.quant_act_2level(dy, both | moss.MOSS_WS_KEPT, out=layer.qdy, workspace=layer.ws_q)
            dx = moss.gemm_fp8_mx(layer.qdy["q_row"], layer.qdy["e_row"], layer.qdy["s"], layer.wq_t, None, layer.s_w)
            moss.gemm_fp8_mx(layer.qdy["q_col"], layer.qdy["e_col"], layer.qdy["s"], layer.qx["q_col"], layer.qx["e_col"],
                             layer.qx["s"], out=layer.dw, out_dtype=torch.float32)
            return dx, None
    return Fn


def _swiglu_fn(moss, torch):
    class Fn(torch.autograd.Function):
        @staticmethod
        def forward(ctx, gate, up, words):
            gate, up = gate.contiguous(), up.contiguous()
            h, word = moss.swiglu_bf16(gate, up)
            ctx.save_for_backward(gate, up)
            ctx.words = words
            if words is not None:
                words.put(h, word)
            return h

        @staticmethod
        def backward(ctx, dh):
            gate, up = ctx.saved_tensors
            dg, du, wg, wu = moss.swiglu_bf16_backward(gate, up, dh.contiguous())
            if ctx.words is not None:
                ctx.words.put(dg, wg)
                ctx.words.put(du, wu)
            return dg, du, None
    return Fn


def _rmsnorm_fns(moss, torch, eps):
    """RMSNorm on the library's kernels: `plain(x, gamma, words)` -> y, and `added(x, delta, gamma, words)` ->
    (h = x + delta, y = norm(h)).  Backward adds the gradient that reaches h over the residual connection inside the
    kernel.  With `words` the maxima of y (forward) and of the gradient (backward) go to the quantizers."""
    class Plain(torch.autograd.Function):
        @staticmethod
        def forward(ctx, x, gamma, words):
            x = x.contiguous()
            _, y, word = moss.add_rmsnorm_bf16(x, gamma, eps)
            ctx.save_for_backward(x, gamma)
            ctx.words = words
            if words is not None:
                words.put(y, word)
            return y

        @staticmethod
        def backward(ctx, dy):
            x, gamma = ctx.saved_tensors
            d, word = moss.rmsnorm_bf16_backward(x, gamma, dy.contiguous(), eps)
            return d, None, None

    class Added(torch.autograd.Function):
        @staticmethod
        def forward(ctx, x, delta, gamma, words):
            h, y, word = moss.add_rmsnorm_bf16(x.contiguous(), gamma, eps, delta=delta.contiguous())
            ctx.save_for_backward(h, gamma)
            ctx.words = words
            if words is not None:
                words.put(y, word)
            return h, y

        @staticmethod
        def backward(ctx, dh, dy):
            h, gamma = ctx.saved_tensors
            d, word = moss.rmsnorm_bf16_backward(h, gamma, dy.contiguous(), eps, d_res=dh.contiguous())
            if ctx.words is not None:
                ctx.words.put(d, word)          # d is the O projection's dY
            return d, d, None, None
    return Plain, Added


class _Bf16Linear:
    def __init__(self, torch, k, n, gen, dev):
        self.master = torch.nn.Parameter(torch.randn((n, k), generator=gen, device=dev, dtype=torch.float32) * 0.02)
        self.master.grad = torch.zeros_like(self.master.data)
        self.w = self.master.data.to(torch.bfloat16)
        self.dw = self.master.grad


def _bf16_linear_fn(torch):
    class Fn(torch.autograd.Function):
        @staticmethod
        def forward(ctx, x, layer):
            ctx.layer = layer
            ctx.save_for_backward(x)
            return x @ layer.w.t()

        @staticmethod
        def backward(ctx, dy):
            (x,) = ctx.saved_tensors
            layer = ctx.layer
            layer.dw.copy_(dy.t() @ x)          # FP32 master gradient from a BF16 GEMM
            return dy @ layer.w, None
    return Fn


class DecoderBlock:
    """hidden -> attention -> SwiGLU FFN, pre-norm, as in LLaMA."""

    def __init__(self, moss, torch, arm, batch, seq, hidden, heads, ffn, seed=5, swiglu="fused", norm="fused"):
        assert arm in ("moss", "bf16") and hidden % heads == 0 and swiglu in ("fused", "torch") and norm in ("fused", "torch")
        self.torch, self.moss, self.arm = torch, moss, arm
        self.words = _MaxWords() if (arm == "moss" and (swiglu == "fused" or norm == "fused")) else None
        self.swiglu = _swiglu_fn(moss, torch) if swiglu == "fused" else None
        self.swiglu_words = self.words if swiglu == "fused" else None
        self.norms = _rmsnorm_fns(moss, torch, 1e-5) if norm == "fused" else None
        self.batch, self.seq, self.hidden, self.heads, self.ffn = batch, seq, hidden, heads, ffn
        dev = torch.device("cuda:0")
        gen = torch.Generator(device=dev)
        gen.manual_seed(seed)
        tokens = batch * seq
        shapes = [("qkv", hidden, 3 * hidden), ("o", hidden, hidden), ("gate", hidden, ffn), ("up", hidden, ffn), ("down", ffn, hidden)]
        if arm == "moss":
            self.lin = {n: _MossLinear(moss, torch, tokens, k, nn, gen, dev, self.words) for n, k, nn in shapes}
            self.fn = _moss_linear_fn(torch)
        else:
            self.lin = {n: _Bf16Linear(torch, k, nn, gen, dev) for n, k, nn in shapes}
            self.fn = _bf16_linear_fn(torch)
            self.opt = torch.optim.AdamW([l.master for l in self.lin.values()], lr=3e-4, betas=(0.9, 0.95), eps=1e-8,
                                         weight_decay=0.1, fused=True)
        bf16 = torch.bfloat16
        self.g1 = torch.ones(hidden, dtype=bf16, device=dev)
        self.g2 = torch.ones(hidden, dtype=bf16, device=dev)
        hd = hidden // heads
        pos = torch.arange(seq, device=dev, dtype=torch.float32)[:, None]
        inv = 1.0 / (10000.0 ** (torch.arange(0, hd, 2, device=dev, dtype=torch.float32) / hd))[None, :]
        ang = torch.cat([pos * inv, pos * inv], dim=1)
        self.cos, self.sin = ang.cos().to(bf16)[None, None], ang.sin().to(bf16)[None, None]
        self.x = torch.randn((batch, seq, hidden), generator=gen, device=dev, dtype=torch.float32).to(bf16)
        self.upstream = (torch.randn((batch, seq, hidden), generator=gen, device=dev, dtype=torch.float32) * 1e-3).to(bf16)
        self.t = 0

    def _rope(self, z):
        hd = z.shape[-1]
        rot = self.torch.cat([-z[..., hd // 2:], z[..., :hd // 2]], dim=-1)
        return z * self.cos + rot * self.sin

    def forward(self, x):
        torch, F = self.torch, self.torch.nn.functional
        B, S, H, nh = self.batch, self.seq, self.hidden, self.heads
        T, hd = B * S, H // nh
        lin, fn = self.lin, self.fn
        xs = x.view(T, H)
        a = self.norms[0].apply(xs, self.g1, self.words) if self.norms else F.rms_norm(xs, (H,), self.g1, 1e-5)
        qkv = fn.apply(a, lin["qkv"]).view(B, S, 3, nh, hd)
        q, k, v = (qkv[:, :, i].transpose(1, 2) for i in range(3))
        att = F.scaled_dot_product_attention(self._rope(q), self._rope(k), v, is_causal=True)
        o = fn.apply(att.transpose(1, 2).reshape(T, H), lin["o"])
        if self.norms:
            h, b = self.norms[1].apply(xs, o, self.g2, self.words)       # residual add and norm in one kernel
        else:
            h = xs + o
            b = F.rms_norm(h, (H,), self.g2, 1e-5)
        if self.swiglu is not None:
            f = self.swiglu.apply(fn.apply(b, lin["gate"]), fn.apply(b, lin["up"]), self.swiglu_words)
        else:
            f = F.silu(fn.apply(b, lin["gate"])) * fn.apply(b, lin["up"])
        return (h + fn.apply(f, lin["down"])).view(B, S, H)

    def train_step(self):
        """forward, backward with the fixed upstream gradient, optimizer step on the five weights"""
        self.t += 1
        if self.words is not None:
            self.words.clear()
        x = self.x.detach().requires_grad_(True)
        out = self.forward(x)
        out.backward(self.upstream)
        if self.arm == "moss":
            for l in self.lin.values():
                l.step(self.t)
        else:
            self.opt.step()
            for l in self.lin.values():
                l.w.copy_(l.master.data)
        return out, x.grad


def attention_flops(batch, seq, hidden, causal=True):
    """matmul FLOPs of attention forward + backward (3.5 x forward), halved for the causal mask"""
    f = 4.0 * batch * seq * seq * hidden
    return 3.5 * f * (0.5 if causal else 1.0)


def linear_flops(batch, seq, hidden, ffn):
    tokens = batch * seq
    return 3 * 2.0 * tokens * (hidden * 3 * hidden + hidden * hidden + 3 * hidden * ffn)


def sizes_small():
    return dict(batch=1, seq=64, hidden=256, heads=2, ffn=512)


def sizes_7b():
    return dict(batch=2, seq=4096, hidden=4096, heads=32, ffn=11008)


__all__ = ["DecoderBlock", "attention_flops", "linear_flops", "sizes_small", "sizes_7b"]
