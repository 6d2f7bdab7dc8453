"""Drop-in PyTorch layer over the SCC C ABI (the paper's third contribution: SCC as a replacement of the
pointwise convolution inside a depthwise-separable block, trainable end to end).

``SCCFunction`` routes autograd through ``scc_forward`` and ``scc_backward`` (or the single-gradient calls when
only one gradient is wanted);
``SCC`` is the module (weight ``[Cout, Cin//cg]``, optional bias).  All SCC arithmetic runs in the HIP kernels;
the bias, which Section 4.2 only mentions among the trainable parameters, is a broadcast add / a sum over
(N, H, W) done with ordinary tensor ops.  Tensors must be CUDA, contiguous NCHW, float32 or bfloat16.

``DWSCCFunction`` / ``DWSCCBlock`` are the whole DW + SCC block (Eq. 2 feeding the SCC of Section 3.1, nothing in
between): the forward is ``scc_dw_forward`` (one fused kernel where the library prefers it), the backward recomputes
the depthwise output, takes ``scc_backward`` on it and hands the result to ``scc_depthwise3x3_backward``.
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


class DWSCCFunction(torch.autograd.Function):
    """y = SCC(DW3x3(x; kdw); weight).  The depthwise output z is not kept between the passes: the fused forward
    never writes it, and the backward recomputes it (one more depthwise stage, a fraction of the block's traffic)
    instead of holding an activation-sized tensor per block."""

    @staticmethod
    def forward(ctx, x, kdw, weight, cg, co, dw_stride):
        x, kdw, weight = x.contiguous(), kdw.contiguous(), weight.contiguous()
        ctx.save_for_backward(x, kdw, weight)
        ctx.cg, ctx.co, ctx.s = int(cg), float(co), int(dw_stride)
        return _scc.scc_dw_forward(x, kdw, weight, ctx.cg, ctx.co, ctx.s)

    @staticmethod
    def backward(ctx, dy):
        x, kdw, weight = ctx.saved_tensors
        dy = dy.contiguous()
        need_x, need_k, need_w = ctx.needs_input_grad[:3]
        z = _scc.scc_depthwise3x3_forward(x, kdw, ctx.s)
        dz = dw = None
        if (need_x or need_k) and need_w:
            dz, dw = _scc.scc_backward(z, dy, weight, ctx.cg, ctx.co)
        elif need_x or need_k:
            dz = _scc.scc_backward_input(dy, weight, z.shape[1], ctx.cg, ctx.co)
        elif need_w:
            dw = _scc.scc_backward_weight(z, dy, ctx.cg, ctx.co)
        dx = dk = None
        if dz is not None:
            dx, dk = _scc.scc_depthwise3x3_backward(x, kdw, dz, ctx.s, need_dx=need_x, need_dk=need_k)
        if dw is not None:
            dw = dw.to(weight.dtype)
        if dk is not None:
            dk = dk.to(kdw.dtype)
        return dx, dk, dw, None, None, None


def dw_scc(x, kdw, weight, cg, co, dw_stride=1, bias=None):
    """Functional form of the block: y = SCC(DW3x3(x; kdw); weight) (+ bias per output channel)."""
    y = DWSCCFunction.apply(x, kdw, weight, cg, co, dw_stride)
    if bias is not None:
        y = y + bias.view(1, -1, 1, 1)
    return y


class DWSCCBlock(torch.nn.Module):
    """Depthwise 3x3 convolution (spatial stride ``stride``, zero padding 1) followed by SCC-cg{cg}-co{co}: the
    paper's replacement of a standard convolution (Sections 2.2 and 3.1), as one trainable module."""

    def __init__(self, in_channels, out_channels, cg=2, co=0.5, stride=1, bias=False, device="cuda", dtype=torch.float32):
        super().__init__()
        L, _, _ = _scc.scc_window_params(in_channels, out_channels, cg, co)
        self.in_channels, self.out_channels, self.cg, self.co, self.stride = in_channels, out_channels, int(cg), float(co), int(stride)
        self.dw_weight = torch.nn.Parameter(torch.empty(in_channels, 3, 3, device=device, dtype=dtype))
        self.weight = torch.nn.Parameter(torch.empty(out_channels, L, device=device, dtype=dtype))
        self.bias = torch.nn.Parameter(torch.zeros(out_channels, device=device, dtype=dtype)) if bias else None
        self.reset_parameters()

    def reset_parameters(self):
        with torch.no_grad():
            self.dw_weight.normal_(0.0, math.sqrt(2.0 / 9.0))                 # He: nine taps per depthwise filter
            self.weight.normal_(0.0, math.sqrt(2.0 / self.weight.shape[1]))
            if self.bias is not None:
                self.bias.zero_()

    def forward(self, x):
        return dw_scc(x, self.dw_weight, self.weight, self.cg, self.co, self.stride, self.bias)

    def extra_repr(self):
        return "%d, %d, cg=%d, co=%g, stride=%d, bias=%s" % (self.in_channels, self.out_channels, self.cg, self.co,
                                                             self.stride, self.bias is not None)
