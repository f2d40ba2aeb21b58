"""The layer as a ``torch.autograd.Function`` and an ``nn.Module`` on top of the C-ABI binding.

Glue only: every arithmetic step of the three passes runs in the library's kernels; torch supplies device memory,
the stream, the autograd graph and (as in the paper, Section 3) the gradient of the bias.  This is the interface the
paper's single-layer measurements use (Section 4.3: ``net.forward(x)`` and ``out.sum().backward()``).
"""
from __future__ import annotations

import torch

from . import binding


class Conv1dFunction(torch.autograd.Function):
    """y = conv1d(x, w[, bias]) with dilation and zero padding; backward = one conv1d_bwd call."""

    @staticmethod
    def forward(ctx, x, w, bias, dilation: int, padding: int, relu: bool, bf16_out: bool):
        x, w = x.contiguous(), w.contiguous()
        ctx.save_for_backward(x, w)
        ctx.geometry = (int(dilation), int(padding))
        ctx.has_bias = bias is not None
        fused = bias is not None or relu or bf16_out
        if fused:
            y = binding.conv1d_fwd_ex(x, w, dilation, padding, bias=None if bias is None else bias.contiguous().float(),
                                      relu=relu, out_bf16=bf16_out)
        else:
            y = binding.conv1d_fwd(x, w, dilation, padding)
        ctx.relu = relu
        if relu:
            ctx.y_positive = y > 0
        return y

    @staticmethod
    def backward(ctx, gy):
        x, w = ctx.saved_tensors
        d, P = ctx.geometry
        if ctx.relu:
            gy = gy * ctx.y_positive
        gb = gy.float().sum(dim=(0, 2)) if ctx.has_bias else None     # the framework's part (Section 3)
        dy = gy.to(x.dtype).contiguous()                               # no copy when the dtypes already agree
        dx, dw = binding.conv1d_bwd(x, dy, w, d, P)
        return dx.to(x.dtype), dw.to(w.dtype), gb, None, None, None, None


def conv1d(x, w, bias=None, dilation: int = 1, padding: int = 0, relu: bool = False, bf16_out: bool = False):
    return Conv1dFunction.apply(x, w, bias, dilation, padding, relu, bf16_out)


class Conv1d(torch.nn.Module):
    """Drop-in for ``torch.nn.Conv1d(C, K, S, dilation=d, padding=P)`` (stride 1, one group) on one MI355X."""

    def __init__(self, in_channels: int, out_channels: int, kernel_size: int, dilation: int = 1, padding: int = 0,
                 bias: bool = False, relu: bool = False, dtype=torch.float32, device="cuda"):
        super().__init__()
        self.dilation, self.padding, self.relu = dilation, padding, relu
        w = torch.empty(out_channels, in_channels, kernel_size, dtype=torch.float32, device=device)
        torch.nn.init.normal_(w, std=(in_channels * kernel_size) ** -0.5)
        self.weight = torch.nn.Parameter(w.to(dtype))
        self.bias = torch.nn.Parameter(torch.zeros(out_channels, dtype=torch.float32, device=device)) if bias else None

    def forward(self, x):
        return conv1d(x, self.weight, self.bias, self.dilation, self.padding, self.relu,
                      bf16_out=False)
