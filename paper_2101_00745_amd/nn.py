"""Drop-in PyTorch layer over the SCC C ABI (the paper's third contribution: SCC as a replacement of the
pointwise convolution inside a depthwise-separable block, trainable end to end).

``SCCFunction`` routes autograd through ``scc_forward`` and ``scc_backward`` (or the single-gradient calls when
only one gradient is wanted);
``SCC`` is the module (weight ``[Cout, Cin//cg]``, optional bias).  All SCC arithmetic runs in the HIP kernels;
the bias, which Section 4.2 only mentions among the trainable parameters, is a broadcast add / a sum over
(N, H, W) done with ordinary tensor ops.  Tensors must be CUDA, contiguous NCHW, float32 or bfloat16.
"""
import math

import torch

from . import scc as _scc


class SCCFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, cg, co):
        x = x.contiguous()
        weight = weight.contiguous()
        ctx.save_for_backward(x, weight)
        ctx.cg, ctx.co = int(cg), float(co)
        return _scc.scc_forward(x, weight, ctx.cg, ctx.co)

    @staticmethod
    def backward(ctx, dy):
        x, weight = ctx.saved_tensors
        dy = dy.contiguous()
        dx = dw = None
        if ctx.needs_input_grad[0] and ctx.needs_input_grad[1]:
            dx, dw = _scc.scc_backward(x, dy, weight, ctx.cg, ctx.co)      # one call, dy and x read once where fused
        elif ctx.needs_input_grad[0]:
            dx = _scc.scc_backward_input(dy, weight, x.shape[1], ctx.cg, ctx.co)
        elif ctx.needs_input_grad[1]:
            dw = _scc.scc_backward_weight(x, dy, ctx.cg, ctx.co)
        if dw is not None:
            dw = dw.to(weight.dtype)                                        # dw comes back as float32
        return dx, dw, None, None


def scc(x, weight, cg, co, bias=None):
    """Functional form: y = SCC(x; weight) (+ bias per output channel)."""
    y = SCCFunction.apply(x, weight, cg, co)
    if bias is not None:
        y = y + bias.view(1, -1, 1, 1)
    return y


class SCC(torch.nn.Module):
    """Sliding-channel convolution SCC-cg{cg}-co{co} from ``in_channels`` to ``out_channels`` (Section 3.1)."""

    def __init__(self, in_channels, out_channels, cg=2, co=0.5, bias=False, device="cuda", dtype=torch.float32):
        super().__init__()
        L, _, _ = _scc.scc_window_params(in_channels, out_channels, cg, co)   # validates (Cin, Cout, cg, co)
        self.in_channels, self.out_channels, self.cg, self.co = in_channels, out_channels, int(cg), float(co)
        self.weight = torch.nn.Parameter(torch.empty(out_channels, L, device=device, dtype=dtype))
        self.bias = torch.nn.Parameter(torch.zeros(out_channels, device=device, dtype=dtype)) if bias else None
        self.reset_parameters()

    def reset_parameters(self):
        L = self.weight.shape[1]
        with torch.no_grad():
            self.weight.normal_(0.0, math.sqrt(2.0 / L))     # He: fan-in of a filter is its window length
            if self.bias is not None:
                self.bias.zero_()

    def forward(self, x):
        return scc(x, self.weight, self.cg, self.co, self.bias)

    def extra_repr(self):
        return "%d, %d, cg=%d, co=%g, bias=%s" % (self.in_channels, self.out_channels, self.cg, self.co,
                                                  self.bias is not None)
