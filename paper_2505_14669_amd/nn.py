"""Drop-in linear layer over the C ABI: forward and backward of Algorithm 1 as one autograd function.

Argument marshalling only: every arithmetic step runs in the library's kernels
(quartet_linear_fwd / quartet_linear_bwd).  torch provides device memory, streams and the autograd
graph.  There is no fallback: without a GPU or without the built library these calls raise.

Shapes: the flattened token count, in_features and out_features must be multiples of the Hadamard
block (32, the MXFP4 group, unless a layer asks for 64, 128 or 256).
"""
import torch

from . import binding as q


class _Workspace:
    """Backward workspace, grown on demand and shared by all layers of a device (calls on one
    stream run one after the other, so one buffer serves them all)."""
    buffers = {}

    @classmethod
    def get(cls, device, nbytes):
        buf = cls.buffers.get(device)
        if buf is None or buf.numel() < nbytes:
            buf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
            cls.buffers[device] = buf
        return buf


class QuartetLinearFunction(torch.autograd.Function):
    """y = x W^T with MXFP4 operands (Algorithm 1 Forward); the backward pass returns the gradients of
    Algorithm 1 Backward.  x: [..., in] bf16, weight: [out, in] bf16, seed: python int naming the
    stochastic-rounding draws of this call's backward pass, rounding: 0 stochastic / 1 nearest,
    hadamard_block: 32 (the method), 64, 128 or 256."""

    @staticmethod
    def forward(ctx, x, weight, seed, rounding, hadamard_block=32):
        if x.dtype != torch.bfloat16 or weight.dtype != torch.bfloat16:
            raise TypeError("QuartetLinearFunction takes bf16 activations and weights")
        if not (x.is_cuda and weight.is_cuda):
            raise RuntimeError("QuartetLinearFunction runs on the GPU only")
        out_f, in_f = weight.shape
        x2 = x.reshape(-1, in_f).contiguous()
        w2 = weight.contiguous()
        tokens = x2.shape[0]
        hb = int(hadamard_block)
        if hb not in (32, 64, 128, 256):
            raise ValueError("hadamard_block must be 32, 64, 128 or 256")
        if tokens % hb or in_f % hb or out_f % hb:
            raise ValueError(f"tokens, in_features and out_features must be multiples of {hb}")
        dev = x.device
        u8 = dict(dtype=torch.uint8, device=dev)
        y = torch.empty((tokens, out_f), dtype=torch.bfloat16, device=dev)
        xq_codes = torch.empty((tokens, in_f // 2), **u8)
        xq_scales = torch.empty((q.quartet_scale_bytes(tokens, in_f),), **u8)
        x_mask = torch.empty((tokens, in_f // 32), dtype=torch.int32, device=dev)
        wq_codes = torch.empty((out_f, in_f // 2), **u8)
        wq_scales = torch.empty((q.quartet_scale_bytes(out_f, in_f),), **u8)
        w_mask = torch.empty((out_f, in_f // 32), dtype=torch.int32, device=dev)
        q.check(q.quartet_linear_fwd_block(x2, w2, tokens, in_f, out_f, hb, y, q.QUARTET_DTYPE_BF16,
                                           xq_codes, xq_scales, x_mask, wq_codes, wq_scales, w_mask))
        ctx.save_for_backward(xq_codes, xq_scales, x_mask, wq_codes, wq_scales, w_mask)
        ctx.dims = (tokens, in_f, out_f, tuple(x.shape), int(seed), int(rounding), hb)
        return y.reshape(*x.shape[:-1], out_f)

    @staticmethod
    def backward(ctx, dy):
        xq_codes, xq_scales, x_mask, wq_codes, wq_scales, w_mask = ctx.saved_tensors
        tokens, in_f, out_f, x_shape, seed, rounding, hb = ctx.dims
        dy2 = dy.reshape(tokens, out_f).to(torch.bfloat16).contiguous()
        dev = dy.device
        dx = torch.empty((tokens, in_f), dtype=torch.bfloat16, device=dev)
        dw = torch.empty((out_f, in_f), dtype=torch.bfloat16, device=dev)
        nbytes = q.quartet_linear_workspace_bytes_block(tokens, in_f, out_f, hb)
        ws = _Workspace.get(dev, nbytes)
        q.check(q.quartet_linear_bwd_block(dy2, tokens, in_f, out_f, hb, xq_codes, xq_scales, x_mask,
                                           wq_codes, wq_scales, w_mask, seed, rounding,
                                           dx, dw, q.QUARTET_DTYPE_BF16, ws, nbytes))
        return dx.reshape(x_shape), dw, None, None, None


class QuartetLinear(torch.nn.Module):
    """nn.Linear replacement: weight [out, in] (bf16, or fp32 master weights cast to bf16 on the way
    in), optional bf16 bias added outside the quantized product.  Every backward pass uses a fresh stochastic-rounding seed: base seed, layer id and a
    per-layer call counter packed into 64 bits, so runs are reproducible and no two calls share draws."""
    _next_id = 0

    def __init__(self, in_features, out_features, bias=False, seed=0, rounding=0, device="cuda",
                 weight_dtype=torch.bfloat16, hadamard_block=32):
        super().__init__()
        self.hadamard_block = hadamard_block
        self.in_features, self.out_features = in_features, out_features
        w = torch.randn(out_features, in_features, device=device) * (in_features ** -0.5)
        # weight_dtype=torch.float32 keeps fp32 master weights; the kernels always see a bf16 copy
        self.weight = torch.nn.Parameter(w.to(weight_dtype))
        self.bias = torch.nn.Parameter(torch.zeros(out_features, dtype=torch.bfloat16, device=device)) if bias else None
        self.rounding = rounding
        self.base_seed = int(seed) & 0xFFFF
        self.layer_id = QuartetLinear._next_id & 0xFFFF
        QuartetLinear._next_id += 1
        self.calls = 0

    def forward(self, x):
        seed = (self.base_seed << 48) | (self.layer_id << 32) | (self.calls & 0xFFFFFFFF)
        self.calls += 1
        y = QuartetLinearFunction.apply(x, self.weight.to(torch.bfloat16), seed, self.rounding, self.hadamard_block)
        return y if self.bias is None else y + self.bias
