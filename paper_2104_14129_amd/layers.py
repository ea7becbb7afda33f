"""Activation-compressed layers (ActNN Sec. 3.2, Eq. (4); Sec. 5.1; Sec. 5.2 levels L2-L4).

A regular layer keeps its full-precision input for the backward pass; an activation-compressed
layer keeps a compressed context instead and computes its gradients from the dequantized
context with the stock backward routine of the layer.  The forward results are those of the
stock layer, so inference is unchanged.

Everything that touches the saved activations runs in libactq through `binding`: per-group
statistics, sensitivities, the device-side bit allocator, quantize + pack, unpack + dequantize,
the ReLU bit mask and the max-pooling positions.  torch supplies the layers' own arithmetic
(GEMM, convolution and batch-norm forward / backward) and the autograd plumbing.  There is no
CPU path: tensors must live on the GPU.
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass

import torch
import torch.nn as nn
import torch.nn.functional as F

from . import binding as B

__all__ = ["QConfig", "config", "set_optimization_level", "compress", "decompress", "SavedContext",
           "QLinear", "QConv2d", "QBatchNorm2d", "QReLU", "QMaxPool2d", "convert"]


@dataclass
class QConfig:
    """How contexts are compressed.

    bits     average code bits per element (the budget of Sec. 4.2's Prob. (9) is bits * N * D)
    mixed    True: per-sample widths from the greedy allocator (level L3); False: every sample
             gets `bits` (an integer 1..8; level L2)
    widths   allowed widths of the allocator (bit b set = b bits)
    header   ACTQ_HDR_F32 or ACTQ_HDR_BF16
    swap     keep the compressed context in pinned host memory between forward and backward (L4)
    seed     Philox key; every saved context draws its own tag from a counter, so no two
             contexts (and no two iterations) share noise
    """
    bits: float = 2.0
    mixed: bool = True
    widths: int = B.ACTQ_WIDTHS_POW2
    header: int = B.ACTQ_HDR_F32
    noise_bits: int = 16
    swap: bool = False
    seed: int = 0


config = QConfig()
_tags = itertools.count(1)
_copy_stream = None


def set_optimization_level(level: str, bits: float | None = None) -> None:
    """L2: per-group quantization at a fixed width; L3: plus per-sample mixed precision; L4: plus
    swapping of the compressed contexts to host memory (Sec. 5.2, Tab. 2).  L0/L1/L5 concern which
    layers are converted and the memory allocator, which are the caller's business here."""
    level = level.upper()
    if level not in ("L2", "L3", "L4"):
        raise ValueError("supported levels: L2, L3, L4")
    config.mixed = level in ("L3", "L4")
    config.swap = level == "L4"
    if bits is not None:
        config.bits = bits


class SavedContext:
    """A compressed activation: bit stream, group headers, per-sample widths and offsets."""

    __slots__ = ("shape", "dtype", "N", "D", "bits", "offsets", "packed", "header", "hf", "host", "ready")

    def nbytes(self) -> int:
        """Bytes held on the device (0 for the streams once they are swapped out)."""
        held = self.bits.numel() + self.offsets.numel() * 8
        for t in (self.packed, self.header):
            if t is not None:
                held += t.numel() * t.element_size()
        return held


_uniform_cache: dict = {}


def _uniform_widths(N: int, D: int, b: int, device):
    key = (N, D, b, device)
    hit = _uniform_cache.get(key)
    if hit is None:
        offsets, total = B.packed_bytes(N, D, [b] * N)
        hit = (torch.full((N,), b, dtype=torch.uint8, device=device),
               torch.from_numpy(offsets.view("int64")).to(device), total)
        _uniform_cache[key] = hit
    return hit


def compress(x: torch.Tensor, grad2: torch.Tensor | None = None) -> SavedContext:
    """Quantize and pack `x` ([N, ...]: the first dimension indexes the samples) under `config`.
    `grad2` are the squared gradient norms per sample of Eq. (8) (None = all ones)."""
    if not x.is_cuda:
        raise ValueError("activation compression runs on the GPU only")
    if x.dtype not in (torch.float32, torch.float16):
        raise TypeError(f"unsupported activation dtype {x.dtype}")
    x = x.contiguous()
    N = int(x.shape[0])
    D = int(x.numel() // N)
    G = B.G_DEFAULT
    ng = (D + G - 1) // G
    c = SavedContext()
    c.shape, c.dtype, c.N, c.D, c.hf, c.host, c.ready = tuple(x.shape), x.dtype, N, D, config.header, None, None
    x2 = x.view(N, D)
    if config.mixed:
        narrowest = min(b for b in range(1, 9) if config.widths >> b & 1)
        if config.bits < narrowest:
            raise ValueError(f"an average of {config.bits} bits is below the narrowest allowed width {narrowest}")
        gmin = torch.empty((N, ng), dtype=torch.float32, device=x.device)
        grange = torch.empty((N, ng), dtype=torch.float32, device=x.device)
        B.group_stats(x2, gmin, grange)
        w = B.sample_sensitivity(grange, grad2)
        budget = int(config.bits * N * D)
        c.bits, c.offsets, _ = B.allocate_bits_device(w, D, budget, config.widths)
        capacity = budget // 8 + N * (ng * G - D) + 32   # the budget in bytes plus the padding of ragged last groups
    else:
        b = int(config.bits)
        if b != config.bits or not 1 <= b <= 8:
            raise ValueError("a fixed width must be an integer from 1 to 8")
        c.bits, c.offsets, capacity = _uniform_widths(N, D, b, x.device)
    c.packed = torch.empty(max(capacity, 32), dtype=torch.uint8, device=x.device)
    c.header = torch.empty(N * ng * 2, dtype=torch.int16 if c.hf == B.ACTQ_HDR_BF16 else torch.float32, device=x.device)
    B.quantize_pack(x2, c.bits, c.offsets, c.packed, c.header, config.seed, next(_tags), config.noise_bits, hf=c.hf)
    if config.swap:
        _swap_out(c)
    return c


def _swap_out(c: SavedContext) -> None:
    """L4: copy the streams to pinned host memory on a side stream and drop the device copies."""
    global _copy_stream
    if _copy_stream is None:
        _copy_stream = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    _copy_stream.wait_stream(main)
    host_packed = torch.empty(c.packed.shape, dtype=c.packed.dtype, pin_memory=True)
    host_header = torch.empty(c.header.shape, dtype=c.header.dtype, pin_memory=True)
    with torch.cuda.stream(_copy_stream):
        host_packed.copy_(c.packed, non_blocking=True)
        host_header.copy_(c.header, non_blocking=True)
        c.packed.record_stream(_copy_stream)
        c.header.record_stream(_copy_stream)
        c.ready = torch.cuda.Event()
        c.ready.record(_copy_stream)
    c.host = (host_packed, host_header)
    c.packed = c.header = None


def decompress(c: SavedContext) -> torch.Tensor:
    """Unpack and dequantize a saved context into a tensor of the original shape and dtype."""
    packed, header = c.packed, c.header
    if c.host is not None:
        torch.cuda.current_stream().wait_event(c.ready)
        packed = c.host[0].to(c.bits.device, non_blocking=True)
        header = c.host[1].to(c.bits.device, non_blocking=True)
    out = torch.empty((c.N, c.D), dtype=c.dtype, device=c.bits.device)
    B.unpack_dequantize(packed, header, c.bits, c.offsets, out, hf=c.hf)
    return out.view(c.shape)


# ----------------------------------------------------------------------------- functions

def _keep(ctx, c: SavedContext, *tensors) -> None:
    """Hands the compressed context to autograd: its tensors are released when the graph is, so a
    second backward pass over a retained graph finds them again."""
    streams = c.host if c.host is not None else (c.packed, c.header)
    ctx.context_meta = (c.shape, c.dtype, c.N, c.D, c.hf, c.ready, c.host is not None)
    ctx.save_for_backward(c.bits, c.offsets, streams[0], streams[1], *tensors)


def _recall(ctx):
    """(dequantized context, the other saved tensors)."""
    bits, offsets, s0, s1, *tensors = ctx.saved_tensors
    c = SavedContext()
    c.shape, c.dtype, c.N, c.D, c.hf, c.ready, swapped = ctx.context_meta
    c.bits, c.offsets = bits, offsets
    c.host, c.packed, c.header = ((s0, s1), None, None) if swapped else (None, s0, s1)
    return decompress(c), tensors


class _QLinearFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias):
        _keep(ctx, compress(x), weight)
        ctx.has_bias = bias is not None
        return F.linear(x, weight, bias)

    @staticmethod
    def backward(ctx, grad_y):
        x, (weight,) = _recall(ctx)
        # under autocast the output (and so grad_y) is narrower than the saved input and the weight:
        # the stock backward then computes in grad_y's type and returns gradients of the operands' types
        g2 = grad_y.reshape(-1, grad_y.shape[-1])
        grad_x = grad_y.matmul(weight.to(grad_y.dtype)).to(x.dtype) if ctx.needs_input_grad[0] else None
        grad_w = (g2.t().matmul(x.reshape(-1, x.shape[-1]).to(grad_y.dtype)).to(weight.dtype)
                  if ctx.needs_input_grad[1] else None)
        grad_b = g2.sum(0).to(weight.dtype) if ctx.has_bias and ctx.needs_input_grad[2] else None
        return grad_x, grad_w, grad_b


class _QConv2dFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, stride, padding, dilation, groups):
        _keep(ctx, compress(x), weight)
        ctx.geometry = (stride, padding, dilation, groups)
        ctx.bias_sizes = None if bias is None else [bias.shape[0]]
        return F.conv2d(x, weight, bias, stride, padding, dilation, groups)

    @staticmethod
    def backward(ctx, grad_y):
        x, (weight,) = _recall(ctx)
        stride, padding, dilation, groups = ctx.geometry
        mask = [ctx.needs_input_grad[0], ctx.needs_input_grad[1], ctx.bias_sizes is not None and ctx.needs_input_grad[2]]
        ct = grad_y.dtype                                # the compute type (narrower under autocast)
        gx, gw, gb = torch.ops.aten.convolution_backward(grad_y.contiguous(), x.to(ct), weight.to(ct), ctx.bias_sizes,
                                                         list(stride), list(padding), list(dilation), False, [0, 0],
                                                         groups, mask)
        return (None if gx is None else gx.to(x.dtype), None if gw is None else gw.to(weight.dtype),
                None if gb is None else gb.to(weight.dtype), None, None, None, None)


class _QBatchNormFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, running_mean, running_var, training, momentum, eps):
        y, mean, invstd = torch.ops.aten.native_batch_norm(x, weight, bias, running_mean, running_var, training,
                                                           momentum, eps)
        _keep(ctx, compress(x), weight, running_mean, running_var, mean, invstd)
        ctx.training, ctx.eps = training, eps
        return y

    @staticmethod
    def backward(ctx, grad_y):
        x, (weight, running_mean, running_var, mean, invstd) = _recall(ctx)
        mask = [ctx.needs_input_grad[0], weight is not None and ctx.needs_input_grad[1],
                weight is not None and ctx.needs_input_grad[2]]
        gx, gw, gb = torch.ops.aten.native_batch_norm_backward(grad_y.contiguous().to(x.dtype), x, weight, running_mean,
                                                               running_var, mean, invstd, ctx.training, ctx.eps, mask)
        return gx, gw, gb, None, None, None, None, None


class _QReLUFn(torch.autograd.Function):
    """Exact: the context is one bit per element."""

    @staticmethod
    def forward(ctx, x):
        y, mask = B.relu_forward(x.contiguous())
        ctx.save_for_backward(mask)
        return y

    @staticmethod
    def backward(ctx, grad_y):
        (mask,) = ctx.saved_tensors
        return B.relu_backward(mask, grad_y.contiguous())


class _QMaxPool2dFn(torch.autograd.Function):
    """Exact: the context is the 8-bit window position of every output location."""

    @staticmethod
    def forward(ctx, x, kernel, stride, padding, dilation):
        y, arg = B.maxpool2d_forward(x.contiguous(), kernel, stride, padding, dilation)
        ctx.save_for_backward(arg)
        ctx.geometry = (int(x.shape[-2]), int(x.shape[-1]), kernel, stride, padding, dilation)
        return y

    @staticmethod
    def backward(ctx, grad_y):
        (arg,) = ctx.saved_tensors
        H, W, kernel, stride, padding, dilation = ctx.geometry
        return B.maxpool2d_backward(arg, grad_y.contiguous(), H, W, kernel, stride, padding, dilation), None, None, None, None


# ----------------------------------------------------------------------------- modules

def _pair(v):
    return (int(v), int(v)) if isinstance(v, int) else (int(v[0]), int(v[1]))


class QLinear(nn.Linear):
    def forward(self, x):
        if torch.is_grad_enabled() and x.is_cuda:
            return _QLinearFn.apply(x, self.weight, self.bias)
        return super().forward(x)


class QConv2d(nn.Conv2d):
    def forward(self, x):
        if torch.is_grad_enabled() and x.is_cuda and self.padding_mode == "zeros" and not isinstance(self.padding, str):
            return _QConv2dFn.apply(x, self.weight, self.bias, self.stride, self.padding, self.dilation, self.groups)
        return super().forward(x)


class QBatchNorm2d(nn.BatchNorm2d):
    def forward(self, x):
        if not (torch.is_grad_enabled() and x.is_cuda and self.training and self.track_running_stats
                and self.momentum is not None):
            return super().forward(x)
        if self.num_batches_tracked is not None:
            self.num_batches_tracked.add_(1)
        return _QBatchNormFn.apply(x, self.weight, self.bias, self.running_mean, self.running_var, True,
                                   self.momentum, self.eps)


class QReLU(nn.Module):
    def forward(self, x):
        if torch.is_grad_enabled() and x.is_cuda and x.dtype in (torch.float32, torch.float16):
            return _QReLUFn.apply(x)
        return F.relu(x)


class QMaxPool2d(nn.MaxPool2d):
    def forward(self, x):
        if (torch.is_grad_enabled() and x.is_cuda and not self.ceil_mode and not self.return_indices
                and x.dtype in (torch.float32, torch.float16)):
            k = _pair(self.kernel_size)
            s = _pair(self.stride if self.stride is not None else self.kernel_size)
            return _QMaxPool2dFn.apply(x, k, s, _pair(self.padding), _pair(self.dilation))
        return super().forward(x)


def convert(module: nn.Module) -> nn.Module:
    """Replace the stock layers of a model by their activation-compressed versions, in place
    (parameters and buffers are shared, not copied)."""
    swaps = {nn.Linear: QLinear, nn.Conv2d: QConv2d, nn.BatchNorm2d: QBatchNorm2d, nn.MaxPool2d: QMaxPool2d}
    for name, child in list(module.named_children()):
        if type(child) is nn.ReLU:
            setattr(module, name, QReLU())
        elif type(child) in swaps:
            child.__class__ = swaps[type(child)]
        else:
            convert(child)
    return module
